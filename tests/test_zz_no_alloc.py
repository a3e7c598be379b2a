"""The allocation-free backward entry point of the attention operator, lx_sparse_attn_bwd_dx_noalloc
(for callers that cannot allocate device memory): host-side errors without a GPU, and on the GPU
its outputs against lx_sparse_attn_bwd_dx's on two calls in a row, the second on a smaller input
(the library-owned scratch still holds the first call's values then)."""
import ctypes as C

import numpy as np
import pytest

from paper_2510_15964_amd import inputs


def _lx():
    from paper_2510_15964_amd import lx
    return lx


def _call(L, B, Hh, S, D, rows_r=None, ptr=0x1000):
    """The entry point with dummy (never dereferenced) pointers: only host-side validation runs."""
    nb = S // 64
    rows = B * 0 + Hh * nb if rows_r is None else rows_r
    bl = L.lx_blocklist(rows, nb, ptr, ptr, rows * nb)
    strides = (C.c_int64 * 3)(Hh * S * D, S * D, D)
    p = C.c_void_p(ptr)
    return L._lib.lx_sparse_attn_bwd_dx_noalloc(L.LX_BF16, B, Hh, S, D, 0.125, 1, p, p, p, p, p, p, strides,
                                                C.byref(bl), C.byref(bl), 1, None, p, p, p, None)


def test_errors_before_any_device_work():
    L = _lx()
    # more (batch, head, token) rows than the library's scratch holds: refused, nothing launched
    assert _call(L, 8, 64, 4096, 64) == L.LX_ERR_WORKSPACE          # 2 097 152 rows > 1 048 576
    assert _call(L, 1, 2, 256, 96) == L.LX_ERR_UNSUPPORTED          # head size
    assert _call(L, 1, 2, 200, 64) == L.LX_ERR_UNSUPPORTED          # S % 64
    assert _call(L, 1, 2, 256, 64, rows_r=3) == L.LX_ERR_INVALID_ARG   # list rows do not match
    assert _call(L, 1, 2, 256, 64, ptr=0x1008) == L.LX_ERR_INVALID_ARG  # misaligned pointers
    assert _call(L, 0, 2, 256, 64) == L.LX_ERR_INVALID_ARG


@pytest.mark.gpu
def test_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    import torch
    from util import dev, host, lx_dtype
    L = _lx()
    assert torch.cuda.is_available()

    def both(c):
        B, Hh, S, D = c["B"], c["Hh"], c["S"], c["D"]
        Q, K, V, dO = (dev(c[k], "bf16") for k in ("Q", "K", "V", "dO"))
        mask = torch.from_numpy(c["mask"]).cuda()
        bl_r, bl_c = L.lx_mask_compact(mask), L.lx_mask_compact(mask, transpose=True)
        ha = torch.from_numpy(c["head_active"]).cuda()
        O = torch.empty_like(Q)
        LSE = torch.empty((B, Hh, S), dtype=torch.float32, device="cuda")
        L.lx_sparse_attn_fwd(Q, K, V, bl_r, c["scale"], c["causal"], O, LSE, mask_batch=c["mask_batch"],
                             head_active=ha)
        ws = torch.empty(L.lx_sparse_attn_bwd_workspace_bytes(lx_dtype(L, "bf16"), B, Hh, S, D),
                         dtype=torch.uint8, device="cuda")
        ref = [torch.full_like(Q, float("nan")) for _ in range(3)]
        L.lx_sparse_attn_bwd_dx(Q, K, V, O, LSE, dO, bl_r, bl_c, c["scale"], c["causal"], *ref, ws,
                                mask_batch=c["mask_batch"], head_active=ha)
        got = [torch.full_like(Q, float("nan")) for _ in range(3)]
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        L.lx_sparse_attn_bwd_dx_noalloc(Q, K, V, O, LSE, dO, bl_r, bl_c, c["scale"], c["causal"], *got,
                                        mask_batch=c["mask_batch"], head_active=ha)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        return [host(t) for t in ref], [host(t) for t in got]

    big = inputs.attn_blocks(2, 4, 512, 64, 0.4, seed=71, dtype="bf16", head_keep=0.75)
    small = inputs.attn_blocks(1, 2, 192, 128, 0.5, seed=72, dtype="bf16")
    for label, c in (("first call", big), ("second, smaller call", small)):
        ref, got = both(c)
        for name, r, g in zip(("dQ", "dK", "dV"), ref, got):
            assert np.isfinite(g).all(), (label, name)
            assert np.array_equal(g, r), (label, name)     # same kernels, same order: same bits
