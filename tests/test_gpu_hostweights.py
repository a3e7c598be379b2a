"""GPU parity: weights kept in CPU memory, only the listed neuron blocks moved to the device
(Sec. VII-B, memory footprint).  The gather is byte work: bit-exact against plain indexing of the
source; the FFN on the gathered blocks equals, bit for bit, the FFN on the full matrices, and the
oracle within the usual gates."""
import numpy as np
import pytest

from paper_2510_15964_amd import inputs
from util import FRO, TOL, dev, host, rel_err_fro, rel_err_max, round_to

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lx():
    import torch
    assert torch.cuda.is_available()
    from paper_2510_15964_amd import lx
    return lx


def _row_list(lx, Fb, nnz, seed, extra_cap=0):
    import torch
    row = np.zeros((1, Fb), np.uint8)
    row[0, np.random.default_rng(seed).choice(Fb, nnz, replace=False)] = 1
    bl = lx.lx_mask_compact(torch.from_numpy(row).cuda(), nnz_cap=nnz + extra_cap)
    return row, bl


@pytest.mark.parametrize("dtype,blk,d,Fb,nnz", [
    ("bf16", 64, 128, 32, 9), ("bf16", 64, 2048, 16, 5), ("f16", 64, 192, 8, 8),
    ("f32", 32, 96, 12, 4), ("f32", 64, 64, 5, 1), ("bf16", 64, 64, 7, 0),
])
@pytest.mark.parametrize("where", ["pinned", "device"])
def test_gather_is_plain_indexing(lx, dtype, blk, d, Fb, nnz, where):
    import torch
    F = Fb * blk
    rng = np.random.default_rng(7 * Fb + nnz)
    W = dev(rng.standard_normal((F, d)).astype(np.float32), dtype)
    src = W.cpu().pin_memory() if where == "pinned" else W
    assert where == "device" or (src.is_pinned() and not src.is_cuda)
    row, bl = _row_list(lx, Fb, nnz, 11 + nnz, extra_cap=3)
    out = torch.full((bl.nnz_cap * blk, d), 7.0, dtype=W.dtype, device="cuda")
    Wc, cl = lx.lx_ffn_gather_weight_blocks(src, bl, blk, out=out)
    torch.cuda.synchronize()
    idx = np.nonzero(row[0])[0]
    want = W.cpu().view(torch.int16 if dtype != "f32" else torch.int32).numpy().reshape(Fb, blk, d)[idx]
    got = Wc.cpu().view(torch.int16 if dtype != "f32" else torch.int32).numpy().reshape(-1, blk, d)
    assert np.array_equal(got[:nnz], want)                       # listed blocks, in list order
    assert (host(Wc).reshape(-1, blk, d)[nnz:] == 7.0).all()     # nothing past the list's end
    assert cl.row_ptr.cpu().tolist() == [0, nnz]
    assert cl.col_idx.cpu().tolist() == list(range(bl.nnz_cap))


@pytest.mark.parametrize("dtype,T,d,Fb,nnz,seed", [
    ("bf16", 512, 128, 24, 7, 31), ("f16", 256, 192, 16, 16, 32), ("bf16", 1024, 256, 40, 12, 33),
])
def test_ffn_on_gathered_blocks_equals_ffn_on_full_weights(lx, oracle, dtype, T, d, Fb, nnz, seed):
    """W_up and W_down_t live in pinned host memory; per call the listed blocks are gathered, the
    two transposes the kernels need are made on the device, and the FFN runs on F' = nnz_cap*64
    neurons with the list 0 .. n-1."""
    import torch
    F = Fb * 64
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, 0.5, seed, dtype=dtype, w_std=0.05)
    row, bl = _row_list(lx, Fb, nnz, seed, extra_cap=min(2, Fb - nnz))
    full = np.repeat(row, T // 64, axis=0)
    X, Wu, Wd, dY = (dev(c[k], dtype) for k in ("X", "W_up", "W_down", "dY"))
    gt = T // 64

    def run(Wu_, Wd_, Wut_, Wdt_, bl_, F_):
        nblocks = bl_.nnz_cap * gt
        ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(lx._dt(X), T, d, F_, 64, 64, nblocks, 1) + 256,
                         dtype=torch.uint8, device="cuda")
        Hd = torch.zeros((nblocks * 4096,), dtype=X.dtype, device="cuda")
        Yd = torch.full_like(X, float("nan"))
        lx.lx_sparse_ffn_fwd(X, Wu_, Wd_, bl_, 64, 64, Yd, Hd)
        dXd = torch.full_like(X, float("nan"))
        lx.lx_sparse_ffn_bwd_dx(dY, Hd, Wu_, Wd_, bl_, 64, 64, dXd, ws, W_up_t=Wut_, W_down_t=Wdt_)
        torch.cuda.synchronize()
        return host(Yd), host(dXd), host(Hd[:nnz * gt * 4096])

    Wut, Wdt = lx.lx_ffn_pack_weights(Wu, Wd)
    Y0, dX0, H0 = run(Wu, Wd, Wut, Wdt, bl, F)
    # host-resident: the two neuron-major matrices
    Wu_h, Wdt_h = Wu.cpu().pin_memory(), Wdt.cpu().pin_memory()
    Wu_c, cl = lx.lx_ffn_gather_weight_blocks(Wu_h, bl, 64)
    Wdt_c, _ = lx.lx_ffn_gather_weight_blocks(Wdt_h, bl, 64)
    Wd_c, Wut_c = lx.lx_ffn_transpose(Wdt_c), lx.lx_ffn_transpose(Wu_c)
    Y1, dX1, H1 = run(Wu_c, Wd_c, Wut_c, Wdt_c, cl, bl.nnz_cap * 64)
    assert np.isfinite(Y1).all() and np.isfinite(dX1).all()
    assert np.array_equal(Y1, Y0) and np.array_equal(dX1, dX0) and np.array_equal(H1, H0)
    H, Y = oracle.ffn_fwd(c["X"], c["W_up"], c["W_down"], full, 64, 64)
    _, dX = oracle.ffn_bwd_dx(c["dY"], c["W_up"], c["W_down"], full, round_to(H, dtype) > 0, 64, 64)
    for g, r in ((Y1, Y), (dX1, dX)):
        assert rel_err_max(g, r) <= TOL[dtype] and rel_err_fro(g, r) <= FRO[dtype]


def test_gather_rejects_what_the_device_cannot_read(lx):
    import torch
    _, bl = _row_list(lx, 8, 3, 1)
    W = torch.zeros((8 * 64, 64), dtype=torch.bfloat16)           # pageable host memory
    with pytest.raises(lx.LxError):
        lx.lx_ffn_gather_weight_blocks(W, bl, 64)
    Wd = W.cuda()
    two_rows = lx.lx_mask_compact(torch.ones((2, 8), dtype=torch.uint8, device="cuda"))
    with pytest.raises(lx.LxError):
        lx.lx_ffn_gather_weight_blocks(Wd, two_rows, 64)           # not a one-row list
    with pytest.raises(lx.LxError):
        lx.lx_ffn_gather_weight_blocks(Wd[:, :40].contiguous(), bl, 32)   # list does not match F / blk_n
    torch.cuda.synchronize()
