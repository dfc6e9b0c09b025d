"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every entry point
the header declares, validates shapes and policies, and reports errors before any launch."""
import ctypes
import os
import re

import pytest

from paper_2411_16786_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dice_moe.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_entry_point():
    names = declared_functions()
    assert {"moe_gate", "moe_dispatch", "moe_expert_ffn", "moe_combine", "moe_conditional_refresh"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own, and a C program that only
    includes it links against the library and reaches the entry points that need no GPU."""
    import subprocess
    src = tmp_path / "use_abi.c"
    src.write_text(
        '#include "dice_moe.h"\n'
        '#include <stdio.h>\n'
        'int main(void) {\n'
        '    moe_shape s = {64, 64, 256, 4, 5, MOE_F32, 0, 0};   /* k > E */\n'
        '    moe_ctx* ctx = 0;\n'
        '    int rc = moe_create(&ctx, &s);\n'
        '    printf("%d %s\\n", rc, moe_status_string(rc));\n'
        '    s.k = 2;\n'
        '    rc = moe_create(&ctx, &s);\n'
        '    printf("%d %lu\\n", rc, (unsigned long)moe_workspace_bytes(ctx));\n'
        '    return moe_destroy(ctx);\n'
        '}\n')
    inc = os.path.dirname(HEADER)
    libdir = os.path.dirname(B.LIB_PATH)
    exe = tmp_path / "use_abi"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, str(src), "-o", str(exe),
                    "-L", libdir, "-ldicemoe", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out[0] == str(B.MOE_ERR_SHAPE) and out[1] == "MOE_ERR_SHAPE"
    assert out[2] == "0" and int(out[3]) >= 64 * 2 * 256 * 4


def test_struct_layouts_match_the_header():
    src = open(HEADER).read()
    shape_fields = re.search(r"typedef struct \{([^{}]*)\} moe_shape;", src, re.S).group(1)
    shape_fields = re.sub(r"/\*.*?\*/", "", shape_fields, flags=re.S)
    names = re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*[,;]", shape_fields)
    assert names == [f[0] for f in B.MoeShape._fields_]
    pol_fields = re.search(r"typedef struct \{([^{}]*)\} moe_policy;", src, re.S).group(1)
    pol_fields = re.sub(r"/\*.*?\*/", "", pol_fields, flags=re.S)
    names = re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*[,;]", pol_fields)
    assert names == [f[0] for f in B.MoePolicy._fields_]


@pytest.mark.parametrize("kw,status", [
    (dict(T_max=64, d=64, F=256, E=4, k=2, dtype="f32"), 0),
    (dict(T_max=64, d=64, F=256, E=4, k=5, dtype="f32"), B.MOE_ERR_SHAPE),       # k > E
    (dict(T_max=64, d=64, F=256, E=65, k=2, dtype="f32"), B.MOE_ERR_SHAPE),      # E > 64
    (dict(T_max=64, d=60, F=256, E=4, k=2, dtype="f32"), B.MOE_ERR_SHAPE),       # d % 16
    (dict(T_max=64, d=96, F=256, E=4, k=2, dtype="bf16"), B.MOE_ERR_SHAPE),      # d % 64 for bf16
    (dict(T_max=-1, d=64, F=256, E=4, k=2, dtype="f32"), B.MOE_ERR_SHAPE),
    (dict(T_max=64, d=4112, F=256, E=4, k=2, dtype="f32"), B.MOE_ERR_SHAPE),     # float rows wider than the router holds
    (dict(T_max=64, d=64, F=256, E=4, k=2, dtype="f32", n_shared=2), 0),
    (dict(T_max=64, d=64, F=256, E=4, k=2, dtype="f32", n_shared=-1), B.MOE_ERR_SHAPE),
    (dict(T_max=64, d=64, F=256, E=63, k=2, dtype="f32", n_shared=2), B.MOE_ERR_SHAPE),  # E + shared > 64
    (dict(T_max=1 << 22, d=2048, F=8192, E=16, k=2, dtype="bf16"), B.MOE_ERR_SHAPE),  # index overflow
])
def test_create_validates_shape(kw, status):
    if status == 0:
        ctx = B.Context(**kw)
        assert ctx.workspace_bytes() >= kw["T_max"] * (kw["k"] + kw.get("n_shared", 0)) * kw["F"] * 4
    else:
        with pytest.raises(B.MoeError) as ei:
            B.Context(**kw)
        assert ei.value.status == status


def test_create_rejects_unknown_dtype_and_null():
    L = B.lib()
    h = ctypes.c_void_p()
    shape = B.MoeShape(64, 64, 256, 4, 2, 7, 0, 0)
    assert L.moe_create(ctypes.byref(h), ctypes.byref(shape)) == B.MOE_ERR_DTYPE
    assert L.moe_create(None, ctypes.byref(shape)) == B.MOE_ERR_NULL
    assert L.moe_destroy(None) == B.MOE_ERR_NULL
    assert L.moe_status_string(B.MOE_ERR_CACHE_COLD) == b"MOE_ERR_CACHE_COLD"


def test_host_detectable_errors_return_before_any_launch():
    L = B.lib()
    ctx = B.Context(T_max=64, d=64, F=256, E=4, k=2, dtype="f32")
    h = ctx._h
    one = ctypes.c_void_p(16)       # a non-null dummy address; never dereferenced on these paths
    # null pointers
    assert L.moe_gate(h, None, one, None, 8, one, one, None, None, None) == B.MOE_ERR_NULL
    assert b"moe_gate" in L.moe_last_error(h)
    # T out of range
    assert L.moe_gate(h, one, one, None, 65, one, one, None, None, None) == B.MOE_ERR_SHAPE
    assert L.moe_dispatch(h, one, one, None, -1, one, one, one, one, one, None, None) == B.MOE_ERR_SHAPE
    # policies
    pol = B.MoePolicy(B.REFRESH_ALG4, 1, 0, 0, 0)
    assert L.moe_conditional_refresh(h, one, one, 8, ctypes.byref(pol), one, one, None, None) == B.MOE_ERR_POLICY
    pol = B.MoePolicy(B.REFRESH_FRACTION_TOKEN, 0, 1, 9, 0)
    assert L.moe_conditional_refresh(h, one, one, 8, ctypes.byref(pol), one, one, None, None) == B.MOE_ERR_POLICY
    pol = B.MoePolicy(B.REFRESH_FRACTION_PAIR, 0, 1, 17, 0)
    assert L.moe_conditional_refresh(h, one, one, 8, ctypes.byref(pol), one, one, None, None) == B.MOE_ERR_POLICY
    pol = B.MoePolicy(99, 0, 1, 0, 0)
    assert L.moe_conditional_refresh(h, one, one, 8, ctypes.byref(pol), one, one, None, None) == B.MOE_ERR_POLICY
    # partial refresh with no cache
    assert L.moe_combine(h, one, one, one, one, 8, None, None, 0, one, None) == B.MOE_ERR_CACHE_COLD
    # FFN: segments, rows, workspace
    assert L.moe_expert_ffn(h, one, one, one, 0, 8, one, None, one, None, one, one, None) == B.MOE_ERR_SHAPE
    assert L.moe_expert_ffn(h, one, one, one, 4, 129, one, None, one, None, one, one, None) == B.MOE_ERR_SHAPE
    assert L.moe_expert_ffn(h, one, one, one, 4, 8, one, None, one, None, one, None, None) == B.MOE_ERR_WORKSPACE
    assert L.moe_expert_ffn_rows(h, one, None, one, one, 4, 8, one, None, one, None, one, one, None) == B.MOE_ERR_NULL
    assert b"row_pairs" in L.moe_last_error(h)
    assert L.moe_expert_ffn_rows(h, one, one, one, one, 4, 129, one, None, one, None, one, one, None) == B.MOE_ERR_SHAPE
    # commit into the pair buffer: (ctx, x_rows, row_pairs, out_pairs, seg_offsets, seg_expert, n_seg, max_rows,
    #                                 W1, b1, W2, b2, scores, mask, T, H_buffer, S_buffer, workspace, stream)
    assert L.moe_expert_ffn_commit(h, one, None, None, one, one, 4, 8, one, None, one, None, one, None, 8, one, one,
                                   one, None) == B.MOE_ERR_NULL                     # no out_pairs
    assert L.moe_expert_ffn_commit(h, one, None, one, one, one, 4, 8, one, None, one, None, one, None, 8, one, None,
                                   one, None) == B.MOE_ERR_NULL                     # no S_buffer
    assert L.moe_expert_ffn_commit(h, one, None, one, one, one, 4, 8, one, None, one, None, one, None, 65, one, one,
                                   one, None) == B.MOE_ERR_SHAPE                    # T > T_max
    assert L.moe_expert_ffn_commit(h, one, None, one, one, one, 4, 8, one, None, one, None, one, None, 8, one, one,
                                   None, None) == B.MOE_ERR_WORKSPACE
    assert L.moe_dispatch(h, None, one, None, 8, one, one, one, one, one, None, None) == B.MOE_ERR_NULL  # rows wanted, no x
    assert L.moe_ep_segments(h, one, 4, 8, one, one, None) == B.MOE_ERR_SHAPE     # E_loc > E
    # T = 0 launches nothing
    assert L.moe_gate(h, one, one, None, 0, one, one, None, None, None) == B.MOE_OK


def test_binding_refuses_cpu_tensors():
    import torch
    ctx = B.Context(T_max=8, d=64, F=256, E=4, k=2, dtype="f32")
    x = torch.zeros(8, 64)
    with pytest.raises(ValueError):
        ctx.moe_gate(x, x, None, x, x)


def test_policy_row_count_matches_the_oracle_mask():
    """moe_policy_refreshed_pairs (the C entry point that sizes the FFN launch from the policy alone,
    without a GPU): the count must equal the number of pairs the oracle's mask (Algorithm 4 and the
    fraction forms) actually refreshes; shared-expert slots add one pair per token in every step."""
    import numpy as np
    from oracle import moe_oracle as O

    rng = np.random.default_rng(7)
    for T, k in ((1, 1), (5, 2), (64, 2), (33, 3)):
        ctx = B.Context(T_max=T, d=64, F=256, E=4, k=k, dtype="f32")
        ctx_shared = B.Context(T_max=T, d=64, F=256, E=4, k=k, dtype="f32", n_shared=2)
        s = rng.random((T, k))
        s = -np.sort(-s, axis=1)            # slot 0 carries the largest score, as the router emits them
        cases = [B.Policy(B.REFRESH_ALL), B.Policy(B.REFRESH_NONE)]
        cases += [B.Policy(kind, step_t=t, stride_n=n, n_units=5) for n in (1, 2, 3) for t in range(4)
                  for kind in (B.REFRESH_ALG4, B.REFRESH_ALG4_HIGH, B.REFRESH_ALG4_RANDOM)]
        cases += [B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=u) for u in (0, 1, T // 2, T)]
        cases += [B.Policy(B.REFRESH_FRACTION_PAIR, n_units=u) for u in (0, 1, T, T * k // 2 + 1, T * k)]
        for pol in cases:
            mask, R = O.refresh_mask(s, pol.kind, pol.step_t, pol.stride_n, pol.n_units)
            assert R == int(mask.sum())
            assert ctx.moe_policy_refreshed_pairs(pol, T) == (R, R), (T, k, pol)
            assert ctx_shared.moe_policy_refreshed_pairs(pol, T) == (R + 2 * T, R)    # shared slots: every token, every step


def test_policy_row_count_rejects_bad_policies():
    ctx = B.Context(T_max=16, d=64, F=256, E=4, k=2, dtype="f32")
    for pol, T in ((B.Policy(B.REFRESH_ALG4, step_t=1, stride_n=0), 8), (B.Policy(B.REFRESH_ALG4, step_t=-1, stride_n=2), 8),
                   (B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=9), 8), (B.Policy(B.REFRESH_FRACTION_PAIR, n_units=17), 8),
                   (B.Policy(99), 8)):
        with pytest.raises(B.MoeError) as e:
            ctx.moe_policy_refreshed_pairs(pol, T)
        assert e.value.status == B.MOE_ERR_POLICY
    with pytest.raises(B.MoeError) as e:
        ctx.moe_policy_refreshed_pairs(B.Policy(B.REFRESH_ALL), 17)      # T beyond T_max
    assert e.value.status == B.MOE_ERR_SHAPE
