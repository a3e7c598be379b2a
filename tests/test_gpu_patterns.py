"""GPU parity: online pattern combination (Sec. VI-A) -- pool layouts + pattern id per head ->
the multi-head block list -- bit-exact against the oracle, and attention under such lists."""
import numpy as np
import pytest

from paper_2510_15964_amd import inputs
from util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lx():
    import torch
    assert torch.cuda.is_available()
    from paper_2510_15964_amd import lx
    return lx


def build_pool(lx, pool):
    """Offline step: the layouts of the pool's patterns (row- and column-compressed)."""
    import torch
    return lx.lx_mask_compact_pair(torch.from_numpy(np.ascontiguousarray(pool)).cuda())


def expected(oracle, pool, hp, transpose):
    m = oracle.combine_patterns(pool, hp)
    if transpose:
        m = m.transpose(0, 2, 1)
    return oracle.mask_compact(m.reshape(-1, m.shape[-1]))


@pytest.mark.parametrize("nblk,heads,causal,seed", [
    (16, 32, True, 1),          # the benchmark's shape
    (5, 7, True, 2),            # ragged sizes
    (33, 300, False, 3),        # more heads than threads of the offset sum, non-causal patterns
    (1, 3, True, 4),            # a single block per head
    (64, 9, True, 5),
])
def test_combine_bit_exact(lx, oracle, nblk, heads, causal, seed):
    import torch
    pool = inputs.pattern_pool(nblk, seed=seed, causal=causal)
    rng = np.random.default_rng(seed)
    hp = rng.integers(-1, pool.shape[0] + 2, heads).astype(np.int32)   # -1 and ids past the pool: no block
    pr, pc = build_pool(lx, pool)
    blr, blc = lx.lx_attn_combine_patterns(pr, pc, nblk, torch.from_numpy(hp).cuda())
    torch.cuda.synchronize()
    for bl, tr in ((blr, False), (blc, True)):
        rp, ci = expected(oracle, pool, hp, tr)
        assert np.array_equal(host(bl.row_ptr), rp)
        assert np.array_equal(host(bl.col_idx)[:rp[-1]], ci)
    # the same lists as compacting the dense multi-head mask on the device
    dense = torch.from_numpy(oracle.combine_patterns(pool, hp)).cuda()
    cr, cc = lx.lx_mask_compact_pair(dense)
    n = int(cr.row_ptr[-1].item())
    assert torch.equal(cr.row_ptr, blr.row_ptr) and torch.equal(cr.col_idx[:n], blr.col_idx[:n])
    assert torch.equal(cc.row_ptr, blc.row_ptr) and torch.equal(cc.col_idx[:n], blc.col_idx[:n])


def test_row_list_only_and_small_capacity(lx, oracle):
    import torch
    pool = inputs.pattern_pool(12, seed=6)
    hp = np.array([7, 0, 3, -1, 5], dtype=np.int32)
    pr, _ = build_pool(lx, pool)
    rp, ci = expected(oracle, pool, hp, False)
    cap = int(rp[-1]) - 40
    blr, blc = lx.lx_attn_combine_patterns(pr, None, 12, torch.from_numpy(hp).cuda(), nnz_cap=cap)
    assert blc is None
    guard = torch.full((cap + 64,), -7, dtype=torch.int32, device="cuda")
    out = (lx.BlockList(5 * 12, 12, blr.row_ptr, guard, cap), None)
    lx.lx_attn_combine_patterns(pr, None, 12, torch.from_numpy(hp).cuda(), nnz_cap=cap, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(host(blr.row_ptr), rp)                       # row_ptr stays exact
    assert np.array_equal(host(guard)[:cap], ci[:cap])                 # the entries that fit
    assert (host(guard)[cap:] == -7).all()                             # nothing past the capacity


def _run_attention(lx, c, blr, blc):
    import torch
    B, Hh, S, D = c["B"], c["Hh"], c["S"], c["D"]
    Q, K, V, dO = (dev(c[k], "bf16") for k in ("Q", "K", "V", "dO"))
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full((B, Hh, S), float("nan"), dtype=torch.float32, device="cuda")
    lx.lx_sparse_attn_fwd(Q, K, V, blr, c["scale"], c["causal"], O, LSE, mask_batch=c["mask_batch"])
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    ws = torch.empty(lx.lx_sparse_attn_bwd_workspace_bytes(lx.LX_BF16, B, Hh, S, D),
                     dtype=torch.uint8, device="cuda")
    lx.lx_sparse_attn_bwd_dx(Q, K, V, O, LSE, dO, blr, blc, c["scale"], c["causal"], dQ, dK, dV, ws,
                             mask_batch=c["mask_batch"])
    torch.cuda.synchronize()
    return dict(O=host(O), LSE=host(LSE), dQ=host(dQ), dK=host(dK), dV=host(dV))


@pytest.mark.parametrize("kw,seed", [
    (dict(B=2, Hh=6, S=512, D=64), 11),
    (dict(B=1, Hh=4, S=320, D=128, head_keep=0.6), 12),
    (dict(B=2, Hh=3, S=256, D=64, mask_batch=2), 13),
    (dict(B=1, Hh=5, S=384, D=64, causal=False), 14),
])
def test_attention_under_combined_lists(lx, oracle, kw, seed):
    """Structured masks (long window rows, global columns) from the pool, through the combination
    kernel, against the oracle run on the dense mask of the same assignment."""
    import torch
    from test_gpu_attn import check, run_oracle
    c = inputs.attn_patterns(seed=seed, **kw)
    nblk = c["S"] // 64
    pr, pc = build_pool(lx, c["pool"])
    blr, blc = lx.lx_attn_combine_patterns(pr, pc, nblk, torch.from_numpy(c["head_pattern"]).cuda())
    got = _run_attention(lx, c, blr, blc)
    mask = oracle.combine_patterns(c["pool"], c["head_pattern"]).reshape(c["mask_batch"], c["Hh"], nblk, nblk)
    ref = run_oracle(oracle, dict(c, mask=mask))
    check(got, ref, f"patterns {kw}")


def test_config3_patterns_full_size_sampled_heads(lx, oracle):
    """The benchmark's pattern workload at full size in its launch configuration; the oracle
    checks sampled (batch, head) pairs."""
    import torch
    from test_gpu_attn import check, run_oracle
    c = inputs.config3_patterns()
    nblk = c["S"] // 64
    pr, pc = build_pool(lx, c["pool"])
    hp = c["head_pattern"]
    blr, blc = lx.lx_attn_combine_patterns(pr, pc, nblk, torch.from_numpy(hp).cuda())
    rp, ci = expected(oracle, c["pool"], hp, False)
    assert np.array_equal(host(blr.row_ptr), rp) and np.array_equal(host(blr.col_idx)[:rp[-1]], ci)
    got = _run_attention(lx, c, blr, blc)
    picks = [(0, 0), (3, int(np.argmax(hp == hp.max()))), (7, c["Hh"] - 1)]
    for (b, h) in picks:
        sub = dict(c, B=1, Hh=1, mask=c["pool"][hp[h]][None, None], head_active=np.ones(1, np.uint8),
                   **{k: c[k][b:b + 1, h:h + 1] for k in ("Q", "K", "V", "dO")})
        check({k: v[b:b + 1, h:h + 1] for k, v in got.items()}, run_oracle(oracle, sub),
              f"config3_patterns b={b} h={h} pattern={hp[h]}")
