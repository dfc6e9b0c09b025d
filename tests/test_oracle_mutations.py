"""Do the pins pin?  One plausible mistake at a time (a transposed operand, a dropped term, a wrong
sign, index, order or constant) is planted in a copy of the oracle's C source; the mutated library is
compiled into a temporary directory and swapped in for the oracle's own, and the pin tests are run
against it.  Every planted mistake must make at least one pin fail.  CPU only; the oracle's source
file and its built library are never touched."""
import ctypes
import inspect
import os
import subprocess

import pytest

import test_oracle_pins as pins
import test_schedule_oracle as schedule_pins
from oracle import moe_oracle as O

SRC = os.path.join(os.path.dirname(O.__file__), "moe_oracle.c")

# (name, text in the source, replacement)
MUTATIONS = [
    ("router operand transposed", "(double)Wg[(size_t)e * d + c]", "(double)Wg[(size_t)c * E + e]"),
    ("router bias subtracted", "if (bg) acc += (double)bg[e];", "if (bg) acc -= (double)bg[e];"),
    ("top-k ties to the higher id", "zi[order[b]] < zi[ea]", "zi[order[b]] <= zi[ea]"),
    ("top-k ascending", "zi[order[b]] < zi[ea]", "zi[order[b]] > zi[ea]"),
    ("softmax not normalised", "for (int e = 0; e < E; ++e) row[e] /= sum;", ""),
    ("renormalisation multiplies", "s[(size_t)i * k + j] /= ssum;", "s[(size_t)i * k + j] *= ssum;"),
    ("Algorithm 4 period inverted", "else if (step_t % stride_n != 0) transmit = 0;",
     "else if (step_t % stride_n == 0) transmit = 0;"),
    ("Algorithm 4 keeps the last slot", "if (j == 0) transmit = 1; ", "if (j == k - 1) transmit = 1; "),
    ("High Score keeps slot 0", "? k - 1\n", "? 0\n"),
    ("ablation period inverted", "(j == fresh_slot) || (step_t % stride_n == 0)",
     "(j == fresh_slot) || (step_t % stride_n != 0)"),
    ("token fraction ranks by the last slot", "it[i].key = s[(size_t)i * k];", "it[i].key = s[(size_t)i * k + k - 1];"),
    ("fraction ranks ascending", "return p->key > q->key ? -1 : 1;", "return p->key < q->key ? -1 : 1;"),
    ("fraction ties to the higher token", "return p->token < q->token ? -1 : 1;", "return p->token > q->token ? -1 : 1;"),
    ("pair fraction fills the last slot first", "return p->slot < q->slot ? -1 : 1;", "return p->slot > q->slot ? -1 : 1;"),
    ("token fraction marks slot 0 only", "for (int j = 0; j < k; ++j) mask[(size_t)it[r].token * k + j] = 1;",
     "mask[(size_t)it[r].token * k] = 1;"),
    ("dispatch in descending pair order",
     "for (size_t p = 0; p < N; ++p)\n            if ((!mask || mask[p]) && idx[p] == e) { perm[r] = (int32_t)p; ++r; }",
     "for (size_t pp = 0; pp < N; ++pp) { size_t p = N - 1 - pp;\n"
     "            if ((!mask || mask[p]) && idx[p] == e) { perm[r] = (int32_t)p; ++r; } }"),
    ("inv of a reused pair is 0", "inv[p] = -1;", "inv[p] = 0;"),
    ("counts ignore the mask", "if (!mask || mask[p]) counts[idx[p]] += 1;", "counts[idx[p]] += 1;"),
    ("packed row taken from the slot number", "(size_t)(perm[r] / k) * d", "(size_t)(perm[r] % k) * d"),
    ("GELU without the square root of two", "erf(u / sqrt(2.0))", "erf(u)"),
    ("GELU by the tanh formula", "0.5 * u * (1.0 + erf(u / sqrt(2.0)))",
     "0.5 * u * (1.0 + tanh(0.7978845608 * (u + 0.044715 * u * u * u)))"),
    ("ReLU instead of GELU", "0.5 * u * (1.0 + erf(u / sqrt(2.0)))", "(u > 0 ? u : 0)"),
    ("W2 transposed", "acc += hidden[f] * (double)w[f];", "acc += hidden[f] * (double)W2e[(size_t)f * d + c];"),
    ("W1 transposed", "u += (double)xrow[c] * (double)w[c];", "u += (double)xrow[c] * (double)W1e[(size_t)c * F + f];"),
    ("b2 dropped", "double acc = b2e ? (double)b2e[c] : 0.0;", "double acc = 0.0;"),
    ("b1 dropped", "double u = b1e ? (double)b1e[f] : 0.0;", "double u = 0.0;"),
    ("segment number used as expert", "const int e = seg_expert[g];", "const int e = g;"),
    ("segment bounds shifted by one", "seg_offsets[g] <= r && r < seg_offsets[g + 1]",
     "seg_offsets[g] < r && r <= seg_offsets[g + 1]"),
    ("reused pair scaled with the wrong score", "ss = use_fresh_scores ? s[p] : S_cache[p];",
     "ss = use_fresh_scores ? S_cache[p] : s[p];"),
    ("no write-through of rows", "if (H_cache) memcpy(H_cache + p * d, hh, sizeof(double) * (size_t)d);", ""),
    ("no write-through of scores", "if (S_cache) S_cache[p] = ss;", ""),
    ("combine reads the neighbouring row", "hh = h_packed + (size_t)inv[p] * d;",
     "hh = h_packed + (size_t)(inv[p] > 0 ? inv[p] - 1 : 0) * d;"),
    ("combine without scores", "yi[c] += ss * hh[c];", "yi[c] += hh[c];"),
    ("combine sums slot 0 only",
     "for (int j = 0; j < k; ++j) {\n            const size_t p = (size_t)i * k + j;\n            const double* hh;",
     "for (int j = 0; j < 1; ++j) {\n            const size_t p = (size_t)i * k + j;\n            const double* hh;"),
    ("receive segment runs the source's number", "seg_expert[g] = el;", "seg_expert[g] = src;"),
    ("receive counts read transposed", "seg_offsets[g + 1] = seg_offsets[g] + recv_counts[g];",
     "seg_offsets[g + 1] = seg_offsets[g] + recv_counts[el * W + src];"),
    ("mixer multiplier", "0x85EBCA6Bu", "0x85EBCA6Du"),
    ("mixer shift", "h ^= h >> 13;", "h ^= h >> 15;"),
    ("mixer seed constant", "seed * 0x9E3779B9u + token", "seed * 0x9E3779B1u + token"),
    ("random slot collapsed to two values", "% (uint32_t)k);", "% (uint32_t)k == 0 ? 0 : 1);"),
]


def _pin_calls():
    """Every pin as a zero-argument callable (a parametrised test once per parameter set)."""
    calls = []
    for mod in (pins, schedule_pins):
        for name, fn in sorted(vars(mod).items(), key=lambda kv: kv[1].__code__.co_firstlineno
                               if inspect.isfunction(kv[1]) else 0):
            if not (name.startswith("test_") and inspect.isfunction(fn)):
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not marks:
                calls.append((name, fn))
                continue
            assert len(marks) == 1 and "," not in marks[0].args[0], "one parameter per pin is all this runner knows"
            for value in marks[0].args[1]:
                calls.append((f"{name}[{value}]", (lambda f=fn, v=value: f(v))))
    return calls


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0].replace(" ", "-") for m in MUTATIONS])
def test_planted_mistake_is_caught_by_a_pin(name, old, new, tmp_path):
    source = open(SRC).read()
    assert source.count(old) >= 1, f"the text to mutate for '{name}' is no longer in the oracle's source"
    mutated_c = tmp_path / "mutant.c"
    mutated_so = tmp_path / "libmutant.so"
    mutated_c.write_text(source.replace(old, new, 1))
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
                           "-std=c11", "-w", "-o", str(mutated_so), str(mutated_c), "-lm"])
    good = O.lib()
    mutant = ctypes.CDLL(str(mutated_so))
    for fn in ("oracle_refresh_mask", "oracle_dispatch", "oracle_combine"):
        getattr(mutant, fn).restype = ctypes.c_int
    failed_pin = None
    O._lib = mutant
    try:
        for pin_name, call in _pin_calls():
            try:
                call()
            except Exception:          # an assertion, or an error the wrong values provoke further on
                failed_pin = pin_name
                break
    finally:
        O._lib = good
    assert failed_pin is not None, f"planted mistake '{name}' passes every pin"


# ---- the schedule oracle (Python): the same check on a copy of its source, run as a module of its own
SCHEDULE_SRC = os.path.join(os.path.dirname(O.__file__), "schedule_oracle.py")

SCHEDULE_MUTATIONS = [
    ("interweaved scales after this step's experts arrived",
     "        y = _scale(st, now.s, pol.use_fresh_scores)\n        # ... the dispatch is waited for within the step, the expert runs on THIS step's rows,\n"
     "        # and its combine is collected in the next step\n        _expert_and_arrive(st, now, routed, E)\n",
     "        _expert_and_arrive(st, now, routed, E)\n        y = _scale(st, now.s, pol.use_fresh_scores)\n"),
    ("displaced experts see this step's dispatch", "_expert_and_arrive(st, st.pending, routed, E)",
     "_expert_and_arrive(st, now, routed, E)"),
    ("displaced scales after the arrival",
     "        y = _scale(st, now.s, pol.use_fresh_scores)\n        _expert_and_arrive(st, st.pending, routed, E)\n",
     "        _expert_and_arrive(st, st.pending, routed, E)\n        y = _scale(st, now.s, pol.use_fresh_scores)\n"),
    ("displaced forgets the new dispatch", "        st.pending = now\n", "        pass\n"),
    ("stale outputs scaled with this step's scores", "s = s_now if use_fresh_scores else st.S",
     "s = st.S if use_fresh_scores else s_now"),
    ("arrived scores not stored", "    Sf[disp.perm] = disp.s.reshape(T * k)[disp.perm]\n", ""),
    ("arrived rows land in packed order", "    Hf[disp.perm] = x_e\n", "    Hf[:len(disp.perm)] = x_e\n"),
    ("shared experts left out of the asynchronous schedules", "        return y + y_shared\n    if schedule == DISPLACED:",
     "        return y\n    if schedule == DISPLACED:"),
    ("shared experts see nothing", "y_shared = O.shared_experts(x, *shared) if n_shared else 0.0", "y_shared = 0.0"),
    ("no synchronous warm-up", "sched = SYNC if (t < warmup or l in sync_layers) else schedule",
     "sched = SYNC if (t < warmup - 1 or l in sync_layers) else schedule"),
    ("Selective Synchronization ignored", "sched = SYNC if (t < warmup or l in sync_layers) else schedule",
     "sched = SYNC if (t < warmup) else schedule"),
    ("no residual between layers", "x = (x.astype(np.float64) + y).astype(np.float32)", "x = y.astype(np.float32)"),
    ("synchronous step leaves no dispatch behind", "        st.pending = Dispatched(r.x_packed, r.offsets, r.perm, r.s, r.mask)",
     "        st.pending = None"),
    ("Algorithm 4 not applied when routing", "mask, _ = O.refresh_mask(s, pol.policy, pol.step_t, pol.stride_n, pol.n_units)",
     "mask, _ = O.refresh_mask(s, O.REFRESH_ALL)"),
]


@pytest.mark.parametrize("name,old,new", SCHEDULE_MUTATIONS, ids=[m[0].replace(" ", "-") for m in SCHEDULE_MUTATIONS])
def test_planted_schedule_mistake_is_caught_by_a_pin(name, old, new):
    import types

    from oracle import schedule_oracle as good
    source = open(SCHEDULE_SRC).read()
    assert source.count(old) >= 1, f"the text to mutate for '{name}' is no longer in the schedule oracle"
    mutant = types.ModuleType("oracle.schedule_oracle_mutant")
    mutant.__package__ = "oracle"
    mutant.__file__ = SCHEDULE_SRC
    import sys
    sys.modules[mutant.__name__] = mutant          # dataclasses look their module up by name
    failed_pin = None
    try:
        exec(compile(source.replace(old, new, 1), SCHEDULE_SRC, "exec"), mutant.__dict__)
        schedule_pins.SO = mutant
        for pin_name, call in _pin_calls():
            if not pin_name.startswith("test_") or getattr(schedule_pins, pin_name.split("[")[0], None) is None:
                continue
            try:
                call()
            except Exception:
                failed_pin = pin_name
                break
    finally:
        schedule_pins.SO = good
        sys.modules.pop(mutant.__name__, None)
    assert failed_pin is not None, f"planted mistake '{name}' passes every schedule pin"
