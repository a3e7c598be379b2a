"""GPU parity: MLP predictor (Sec. V-A) -- block scores, threshold, OR over token groups --
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from paper_2510_15964_amd import inputs
from util import dev, host, round_to

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lx():
    import torch
    assert torch.cuda.is_available()
    from paper_2510_15964_amd import lx
    return lx


def _case(T, d, nblk, seed, dtype="bf16"):
    rng = np.random.default_rng(seed)
    X = round_to(rng.standard_normal((T, d)), dtype)
    Wa_t = round_to(rng.standard_normal((nblk, d)) / np.sqrt(d), dtype)
    return X, Wa_t


def _check(lx, oracle, X, Wa_t, thr, group, dtype="bf16"):
    """The decision is made on fp32 sums of bf16 products on the GPU and in fp64 in the oracle:
    both must agree wherever the oracle's scores of a (group, block) are not within rounding
    distance of the threshold; inside that band either value is valid."""
    import torch
    T, d = X.shape
    nblk = Wa_t.shape[0]
    S, M = oracle.mlp_predict(X, np.ascontiguousarray(Wa_t.T), thr, group_rows=group)
    got = host(lx.lx_mlp_predict_mask(dev(X, dtype), dev(Wa_t, dtype), float(thr), group))
    assert got.shape == M.shape and set(np.unique(got)) <= {0, 1}
    # fp32 accumulation of d products of magnitude |x||w|: a few ulp of the running sum
    band = 4 * np.finfo(np.float32).eps * np.sqrt(d) * (np.abs(X).astype(np.float64) @ np.abs(Wa_t.T).astype(np.float64)).max()
    G = T // group
    Sg = S.reshape(G, group, nblk)
    near = (np.abs(Sg - thr) <= band).any(axis=1)            # some token of the group is ambiguous
    clear = ~near | (Sg > thr + band).any(axis=1)            # ...unless another token decides it anyway
    assert np.array_equal(got[clear], M[clear])
    assert clear.mean() > 0.99
    return got, M


@pytest.mark.parametrize("T,d,nblk,group,thr,seed", [
    (256, 128, 64, 64, 2.5, 1),          # one mask row per token tile
    (512, 256, 128, 512, 3.1, 2),        # one row for all tokens (the paper's reduction)
    (512, 192, 320, 128, 2.5, 3),        # nblk = 5 groups of 64: a ragged last chunk of the pipeline
    (64, 64, 64, 64, 2.2, 4),            # smallest shape
    (2048, 128, 2048, 256, 2.8, 6),      # enough work for workgroups of four 64-row groups of Wa_t
    (8192, 64, 384, 1024, 3.2, 7),       # ... of two (6 groups of rows, 128 token tiles)
])
def test_predict_matches_oracle(lx, oracle, T, d, nblk, group, thr, seed):
    X, Wa_t = _case(T, d, nblk, seed)
    got, M = _check(lx, oracle, X, Wa_t, thr, group)
    assert 0.02 < M.mean() < 0.98                             # the case is not degenerate


def test_threshold_limits(lx, oracle):
    import torch
    X, Wa_t = _case(256, 128, 128, 5)
    lo = host(lx.lx_mlp_predict_mask(dev(X, "bf16"), dev(Wa_t, "bf16"), -1e30, 256))
    hi = host(lx.lx_mlp_predict_mask(dev(X, "bf16"), dev(Wa_t, "bf16"), 1e30, 256))
    assert lo.all() and not hi.any()


def test_predicted_mask_feeds_the_sparse_ffn(lx, oracle):
    """Predictor -> compaction -> sparse FFN with one list shared by all tokens: the chain the
    paper runs per layer; checked against the oracle run on the oracle's own mask."""
    import torch
    from util import FRO, TOL, rel_err_fro, rel_err_max
    T, d, F = 512, 256, 4096
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, 0.5, 91, dtype="bf16", w_std=0.05)
    nblk = F // 64
    rng = np.random.default_rng(92)
    Wa_t = inputs.bf16_round((rng.standard_normal((nblk, d)) / np.sqrt(d)).astype(np.float32))
    thr = 3.1
    S, M = oracle.mlp_predict(c["X"], np.ascontiguousarray(Wa_t.T), thr)
    assert 0 < M.sum() < nblk
    assert np.abs(S - thr).min() > 1e-3                       # no score near the threshold here
    X, Wu, Wd = (dev(c[k], "bf16") for k in ("X", "W_up", "W_down"))
    mask = lx.lx_mlp_predict_mask(X, dev(Wa_t, "bf16"), thr, T)
    assert np.array_equal(host(mask), M)
    bl = lx.lx_mask_compact(mask)
    Y = torch.full_like(X, float("nan"))
    H = torch.empty(bl.nnz_cap * (T // 64) * 4096, dtype=X.dtype, device="cuda")
    lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, 64, 64, Y, H)
    torch.cuda.synchronize()
    _, Yref = oracle.ffn_fwd(c["X"], c["W_up"], c["W_down"], np.repeat(M, T // 64, axis=0), 64, 64)
    assert rel_err_max(host(Y), Yref) <= TOL["bf16"] and rel_err_fro(host(Y), Yref) <= FRO["bf16"]


def test_shared_list_full_size_sampled_tiles(lx, oracle):
    """The benchmark's workload at the paper's operating point (T = 4096, d = 2048, F = 8192, one
    predicted list of 11 % of the blocks for all tokens) in the launch configuration bench.py times:
    mask bit-exact against the oracle's predictor, forward and input gradient on sampled token tiles
    (tiles are independent given the list)."""
    import torch
    from util import FRO, TOL, compact_blocks, rel_err_fro, rel_err_max
    T, d, F, Tt = 4096, 2048, 8192, 64
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, 0.11, seed=2100, dtype="bf16")
    p = inputs.predictor_planted(d, F // 64, 0.11, seed=2100)
    S, M = oracle.mlp_predict(c["X"], np.ascontiguousarray(p["Wa_t"].T), p["thr"])
    assert np.array_equal(M[0].astype(bool), p["hot"])
    band = 4 * np.finfo(np.float32).eps * np.sqrt(d) * (np.abs(c["X"]).astype(np.float64) @ np.abs(p["Wa_t"].T).astype(np.float64)).max()
    hi = S.max(axis=0)                                        # the token that decides each block
    assert (np.abs(hi - p["thr"]) > band).all()               # no block is decided inside the rounding band
    X, Wu, Wd, dY = (dev(c[k], "bf16") for k in ("X", "W_up", "W_down", "dY"))
    mask = lx.lx_mlp_predict_mask(X, dev(p["Wa_t"], "bf16"), p["thr"], T)
    assert np.array_equal(host(mask), M)
    bl = lx.lx_mask_compact(mask)
    n = int(M.sum())
    assert bl.rows == 1 and int(bl.row_ptr[-1].item()) == n
    H = torch.full((bl.nnz_cap * Tt * 4096,), float("nan"), dtype=X.dtype, device="cuda")
    Y = torch.full_like(X, float("nan"))
    lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, 64, 64, Y, H)
    Wut, Wdt = lx.lx_ffn_pack_weights(Wu, Wd)
    ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(lx.LX_BF16, T, d, F, 64, 64, bl.nnz_cap * Tt, 1),
                     dtype=torch.uint8, device="cuda")
    dX = torch.full_like(X, float("nan"))
    lx.lx_sparse_ffn_bwd_dx(dY, H, Wu, Wd, bl, 64, 64, dX, ws, W_up_t=Wut, W_down_t=Wdt)
    torch.cuda.synchronize()
    Hh = host(H[:n * Tt * 4096]).reshape(n, Tt, 64, 64)       # [entry][tile][token][neuron]
    Yh, dXh = host(Y), host(dX)
    assert np.isfinite(Hh).all() and np.isfinite(Yh).all() and np.isfinite(dXh).all()
    cols = np.nonzero(M[0])[0]
    for i in (0, 29, 63):
        sl = slice(i * 64, (i + 1) * 64)
        Href, Yref = oracle.ffn_fwd(c["X"][sl], c["W_up"], c["W_down"], M, 64, 64)
        gate = np.zeros((64, F), dtype=bool)                  # the stored activations decide the gate
        for k, j in enumerate(cols):
            gate[:, j * 64:(j + 1) * 64] = Hh[k, i] > 0
        _, dXref = oracle.ffn_bwd_dx(c["dY"][sl], c["W_up"], c["W_down"], M, gate, 64, 64)
        prs = ((Hh[:, i], compact_blocks(Href, M, 64, 64)), (Yh[sl], Yref), (dXh[sl], dXref))
        errs, fro = [rel_err_max(*q) for q in prs], [rel_err_fro(*q) for q in prs]
        print(f"shared list, tile {i}: max-rel {errs} fro {fro}", flush=True)
        assert max(errs) <= TOL["bf16"] and max(fro) <= FRO["bf16"]
