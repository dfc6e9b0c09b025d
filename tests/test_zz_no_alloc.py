"""moe_dispatch_noalloc (the entry point for callers that cannot allocate or pass a workspace: its
scratch is a device array inside the library) against moe_dispatch, through the C-ABI: the same
outputs bit for bit, on calls in a row that share the one static array."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2411_16786_amd import binding as B
from paper_2411_16786_amd import workloads as WL

import gpu_util as G

pytestmark = pytest.mark.gpu


def run_both(ctx, T, E, k, d, seed, masked):
    r = np.random.Generator(np.random.PCG64(seed))
    x = G.to_dev(WL.to_storage(r.standard_normal((T, d), dtype=np.float32), "bf16"), "bf16")
    idx = O.topk(r.standard_normal((T, E)) + np.log(WL.zipf_weights(E, 1.2)), k)
    mask = (r.random((T, k)) < 0.6).astype(np.uint8) if masked else None
    idx_dev = G.i32_dev(idx)
    mask_dev = None if mask is None else G.u8_dev(mask)
    N = T * k
    out = []
    for which in ("workspace", "static"):
        xp = torch.full((N, d), -3.0, dtype=torch.bfloat16, device=G.DEV)
        counts = torch.full((E,), -9, dtype=torch.int32, device=G.DEV)
        offsets = torch.full((E + 1,), -9, dtype=torch.int32, device=G.DEV)
        perm = torch.full((N,), -9, dtype=torch.int32, device=G.DEV)
        inv = torch.full((N,), -9, dtype=torch.int32, device=G.DEV)
        if which == "workspace":
            ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
            ctx.moe_dispatch(x, idx_dev, mask_dev, xp, counts, offsets, perm, inv, ws)
        else:
            ctx.moe_dispatch_noalloc(x, idx_dev, mask_dev, xp, counts, offsets, perm, inv)
        torch.cuda.synchronize()
        out.append([G.to_np(t) for t in (xp, counts, offsets, perm, inv)])
    # the reference entry point is itself held to the oracle
    c_ref, o_ref, p_ref, i_ref = O.dispatch(idx, mask, E)
    np.testing.assert_array_equal(out[0][1], c_ref)
    np.testing.assert_array_equal(out[0][3][:p_ref.shape[0]], p_ref)
    for a, b_, name in zip(out[0], out[1], ("x_packed", "counts", "offsets", "perm", "inv")):
        np.testing.assert_array_equal(a, b_, err_msg=f"{name}: T={T}")
    return int(o_ref[-1])


def test_dispatch_noalloc_matches_dispatch_on_calls_in_a_row():
    E, k, d = 8, 2, 64
    ctx = B.Context(20000, d, 64, E, k, "bf16")
    # large first (157 workgroups' counts in the static array), then smaller ones that reuse its front,
    # then a single-workgroup call that needs no scratch, then large again
    for T, masked, seed in ((20000, True, 1), (3000, True, 2), (1500, False, 3), (700, True, 4), (20000, False, 5)):
        print(f"moe_dispatch_noalloc T={T} masked={masked}", flush=True)
        R = run_both(ctx, T, E, k, d, seed, masked)
        assert 0 < R <= T * k


def test_dispatch_noalloc_rejects_sizes_beyond_its_static_scratch():
    E, k, d, T = 64, 2, 64, 300000          # 293 workgroups x 64 experts x 4 bytes > 64 KiB
    ctx = B.Context(T, d, 64, E, k, "bf16")
    N = T * k
    idx = torch.zeros((T, k), dtype=torch.int32, device=G.DEV)
    counts = torch.full((E,), -9, dtype=torch.int32, device=G.DEV)
    offsets = torch.full((E + 1,), -9, dtype=torch.int32, device=G.DEV)
    perm = torch.full((N,), -9, dtype=torch.int32, device=G.DEV)
    inv = torch.full((N,), -9, dtype=torch.int32, device=G.DEV)
    with pytest.raises(B.MoeError) as e:
        ctx.moe_dispatch_noalloc(None, idx, None, None, counts, offsets, perm, inv)
    assert e.value.status == B.MOE_ERR_SHAPE and "static buffer" in str(e.value)
    torch.cuda.synchronize()
    assert (counts == -9).all() and (perm == -9).all()          # nothing was launched
