"""GPU parity: sparse FFN forward and input gradient against the CPU oracle,
called through the C ABI (ctypes binding)."""
import numpy as np
import pytest

from paper_2510_15964_amd import inputs
import emulate16
from util import (FRO, TOL, assert_within_emulated, compact_blocks, dev, host, rel_err, rel_err_fro,
                  rel_err_max, round_to, lx_dtype)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lx():
    import torch
    assert torch.cuda.is_available()
    from paper_2510_15964_amd import lx
    return lx


def run_gpu(lx, c, mask=None, packed=True, bias=False, h_from=None):
    """Returns dict of host arrays: Y, H_act (compact), dX, and the list."""
    import torch
    mask = c["mask"] if mask is None else mask
    dt, tt, bn = c["dtype"], c["tile_t"], c["blk_n"]
    T, d, F = c["T"], c["d"], c["F"]
    X, Wu, Wd, dY = (dev(c[k], dt) for k in ("X", "W_up", "W_down", "dY"))
    bu = dev(c["b_up"], dt) if bias else None
    bd = dev(c["b_down"], dt) if bias else None
    m = torch.from_numpy(np.ascontiguousarray(mask)).cuda()
    bl = lx.lx_mask_compact(m)
    cap = bl.nnz_cap
    tdt = X.dtype
    guard = 4096
    H_act = torch.full((cap * tt * bn + guard,), float("nan"), dtype=tdt, device="cuda")
    Y = torch.full((T, d), float("nan"), dtype=tdt, device="cuda")
    lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, tt, bn, Y, H_act, b_up=bu, b_down=bd)
    nnz = int(bl.row_ptr[-1].item())
    out = dict(Y=host(Y), H_act=host(H_act[:nnz * tt * bn]).reshape(nnz, tt, bn), nnz=nnz)
    assert torch.isnan(H_act[cap * tt * bn:]).all(), "wrote past the H_act buffer"
    if h_from is not None:                      # backward consumes a supplied activation buffer
        H_in = torch.zeros_like(H_act)
        H_in[:nnz * tt * bn] = dev(h_from.reshape(-1), dt)
    else:
        H_in = H_act
    dtc = lx_dtype(lx, dt)
    ws_bytes = lx.lx_sparse_ffn_bwd_workspace_bytes(dtc, T, d, F, tt, bn, cap, 1 if packed else 0)
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    dX = torch.full((T, d), float("nan"), dtype=tdt, device="cuda")
    if packed:
        Wut, Wdt = lx.lx_ffn_pack_weights(Wu, Wd)
        bits = torch.int32 if dt == "f32" else torch.int16        # bit compare (NaN-safe)
        assert torch.equal(Wut.view(bits), Wu.t().contiguous().view(bits))
        assert torch.equal(Wdt.view(bits), Wd.t().contiguous().view(bits))
        lx.lx_sparse_ffn_bwd_dx(dY, H_in, Wu, Wd, bl, tt, bn, dX, ws, W_up_t=Wut, W_down_t=Wdt)
    else:
        lx.lx_sparse_ffn_bwd_dx(dY, H_in, Wu, Wd, bl, tt, bn, dX, ws)
    torch.cuda.synchronize()
    out["dX"] = host(dX)
    return out


def run_oracle(oracle, c, mask=None, bias=False):
    mask = c["mask"] if mask is None else mask
    dt, tt, bn = c["dtype"], c["tile_t"], c["blk_n"]
    H, Y = oracle.ffn_fwd(c["X"], c["W_up"], c["W_down"], mask, tt, bn,
                          c["b_up"] if bias else None, c["b_down"] if bias else None)
    # the backward pass takes the stored activations as input: both sides use the
    # oracle's H rounded to the run dtype, so the ReLU gate is decided once
    Hq = round_to(H, dt)
    dZ, dX = oracle.ffn_bwd_dx(c["dY"], c["W_up"], c["W_down"], mask, Hq > 0, tt, bn)
    out = dict(H=H, Y=Y, dX=dX, Hq_act=compact_blocks(Hq, mask, tt, bn),
               H_act=compact_blocks(H, mask, tt, bn))
    if dt != "f32":
        # the ideal 16-bit pipeline on the same input: what the element-wise gate is derived from
        em = emulate16.ffn(c, mask, c["b_up"] if bias else None, c["b_down"] if bias else None,
                           act=Hq > 0)
        out["emul"] = dict(H=compact_blocks(em["H"], mask, tt, bn), Y=em["Y"], dX=em["dX"])
    return out


def compare(lx, oracle, c, mask=None, packed=True, bias=False):
    ref = run_oracle(oracle, c, mask, bias)
    got = run_gpu(lx, c, mask, packed, bias, h_from=ref["Hq_act"])
    tol = TOL[c["dtype"]]
    assert got["nnz"] == int(np.count_nonzero(c["mask"] if mask is None else mask))
    pairs = dict(H=(got["H_act"], ref["H_act"]), Y=(got["Y"], ref["Y"]), dX=(got["dX"], ref["dX"]))
    errs = {k: rel_err_max(*v) for k, v in pairs.items()}
    fro = {k: rel_err_fro(*v) for k, v in pairs.items()}
    floor = {k: rel_err(*v) for k, v in pairs.items()}
    print(f"[{c['dtype']} T={c['T']} d={c['d']} F={c['F']} nnz={got['nnz']}] max-rel {errs} "
          f"fro {fro} rms-floored {floor}", flush=True)
    for k in pairs:
        assert errs[k] <= tol, (k, errs[k], tol)
        assert fro[k] <= FRO[c["dtype"]], (k, fro[k])
        if c["dtype"] == "f32":          # fp32 meets the element-wise gate as it stands
            assert floor[k] <= tol, (k, floor[k])
        elif pairs[k][1].size:           # 16-bit: at most a quarter above the ideal 16-bit pipeline
            assert_within_emulated(*pairs[k], ref["emul"][k], k)
    assert np.isfinite(got["Y"]).all() and np.isfinite(got["dX"]).all()
    return got, ref


def test_config1_fp32_full(lx, oracle):
    """configs[0]: OPT-125m-shaped FFN, fp32, 32x32 blocks, 30 % density."""
    compare(lx, oracle, inputs.config1_ffn())


@pytest.mark.parametrize("tile,T,d,F,density,seed", [
    (32, 96, 64, 160, 0.5, 1), (64, 192, 96, 320, 0.4, 2), (64, 128, 32, 64, 1.0, 3),
    (32, 64, 32, 96, 0.0, 4),
])
def test_fp32_small_shapes(lx, oracle, tile, T, d, F, density, seed):
    c = inputs.ffn_bernoulli(T, d, F, tile, tile, density, seed, dtype="f32", w_std=0.1)
    compare(lx, oracle, c)
    compare(lx, oracle, c, packed=False)


@pytest.mark.parametrize("T,d,F,density,seed", [
    (256, 256, 1024, 0.3, 11),      # several tiles, ragged per-row counts
    (192, 192, 704, 0.45, 12),      # d not a multiple of 256, 11 neuron blocks
    (128, 64, 320, 1.0, 13),        # dense
    (128, 128, 256, 0.0, 14),       # empty mask
    (64, 576, 64, 1.0, 15),         # single block
])
def test_bf16_small_shapes(lx, oracle, T, d, F, density, seed):
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, density, seed, dtype="bf16", w_std=0.05)
    compare(lx, oracle, c)
    compare(lx, oracle, c, packed=False)


@pytest.mark.parametrize("dtype,tile", [("f32", 32), ("bf16", 64)])
def test_bias_and_rows_without_blocks(lx, oracle, dtype, tile):
    c = inputs.ffn_bernoulli(4 * tile, 128, 8 * tile, tile, tile, 0.4, 21, dtype=dtype, w_std=0.1)
    rng = np.random.default_rng(3)
    c["b_up"] = round_to(rng.standard_normal(c["F"]) * 0.1, dtype)
    c["b_down"] = round_to(rng.standard_normal(c["d"]), dtype)
    c["mask"][1, :] = 0                       # a token tile with no active block
    c["mask"][2, :] = [1, 0, 0, 0, 0, 1, 1, 1]
    got, ref = compare(lx, oracle, c, bias=True)
    sl = slice(tile, 2 * tile)
    assert np.array_equal(got["Y"][sl], np.broadcast_to(c["b_down"], (tile, c["d"])))
    assert not got["dX"][sl].any()
    got, ref = compare(lx, oracle, c, bias=False)
    assert not got["Y"][sl].any()


def test_inactive_weight_blocks_are_never_read(lx, oracle):
    """Sec. II-D on the GPU: NaN in every weight block that no token tile uses."""
    c = inputs.ffn_bernoulli(256, 128, 1024, 64, 64, 0.3, 31, dtype="bf16", w_std=0.05)
    c["mask"][:, [2, 5, 11]] = 0
    ref = run_gpu(lx, c)
    c2 = dict(c, W_up=c["W_up"].copy(), W_down=c["W_down"].copy())
    for j in (2, 5, 11):
        c2["W_up"][j * 64:(j + 1) * 64] = np.nan
        c2["W_down"][:, j * 64:(j + 1) * 64] = np.nan
    for packed in (True, False):
        got = run_gpu(lx, c2, packed=packed)
        for k in ("Y", "H_act", "dX"):
            assert np.array_equal(got[k], ref[k]), k


def test_forward_backward_chain_on_device(lx, oracle):
    """fwd -> bwd with the device's own H_act (the normal call sequence)."""
    c = inputs.ffn_bernoulli(256, 128, 512, 64, 64, 0.5, 41, dtype="bf16", w_std=0.05)
    got = run_gpu(lx, c)
    ref = run_oracle(oracle, c)
    flips = int(np.count_nonzero((got["H_act"] > 0) != (ref["Hq_act"] > 0)))
    print("gate flips between device and oracle activations:", flips, flush=True)
    if flips == 0:
        assert rel_err_max(got["dX"], ref["dX"]) <= TOL["bf16"]


def test_planted_support_mask_equals_dense_on_device(lx, oracle):
    """Mask = true ReLU support: the sparse result must equal the dense one."""
    c = inputs.ffn_planted_support(512, 256, 2048, 64, 64, 0.5, 4.0, seed=51)
    sparse = run_gpu(lx, c)
    dense = run_gpu(lx, c, mask=np.ones_like(c["mask"]))
    # same products, only all-zero blocks are skipped; accumulation order over
    # blocks is ascending in both, so Y agrees to rounding of skipped zeros: exactly
    assert np.array_equal(sparse["Y"], dense["Y"])
    assert np.array_equal(sparse["dX"], dense["dX"])
    ref = run_oracle(oracle, c)
    assert rel_err_max(sparse["Y"], ref["Y"]) <= TOL["bf16"]


def test_config2_bf16_full_size_sampled_tiles(lx, oracle):
    """configs[1] at full size in the benchmark's launch configuration; the
    oracle checks sampled token tiles (tiles are independent)."""
    c = inputs.config2_ffn()
    got = run_gpu(lx, c)
    assert got["nnz"] == int(c["mask"].sum())
    rp = np.concatenate([[0], np.cumsum(c["mask"].sum(1, dtype=np.int64))]).astype(np.int64)
    for i in (0, 17, 63):
        sl = slice(i * 64, (i + 1) * 64)
        sub = dict(c, X=c["X"][sl], dY=c["dY"][sl], mask=c["mask"][i:i + 1], T=64)
        ref = run_oracle(oracle, sub)
        Hg = got["H_act"][rp[i]:rp[i + 1]]
        # backward of the sampled tile with the oracle's activations
        sub_got = run_gpu(lx, sub, h_from=ref["Hq_act"])
        prs = ((Hg, ref["H_act"]), (got["Y"][sl], ref["Y"]), (sub_got["dX"], ref["dX"]))
        errs = [rel_err_max(*p) for p in prs]
        fro = [rel_err_fro(*p) for p in prs]
        print(f"config2 tile {i}: n_active={int(c['mask'][i].sum())} max-rel {errs} fro {fro} "
              f"rms-floored {[rel_err(*p) for p in prs]}", flush=True)
        assert max(errs) <= TOL["bf16"] and max(fro) <= FRO["bf16"]
        for name, p in zip(("H", "Y", "dX"), prs):
            assert_within_emulated(*p, ref["emul"][name], name)
        # full-size launch and single-tile launch agree bit for bit on this tile
        assert np.array_equal(sub_got["Y"], got["Y"][sl])
    # tiles with no active block are exactly zero
    for i in np.nonzero(c["mask"].sum(1) == 0)[0]:
        assert not got["Y"][i * 64:(i + 1) * 64].any()


@pytest.mark.parametrize("dtype,tile", [("f32", 32), ("bf16", 64)])
def test_list_longer_than_its_capacity_is_truncated(lx, dtype, tile):
    """A capacity bound that was too small: the entries after the first nnz_cap (list order)
    are ignored by every call, nothing past the buffers is written, and the results are
    bit-identical to those of the truncated mask."""
    import torch
    c = inputs.ffn_bernoulli(4 * tile, 256, 8 * tile, tile, tile, 0.4, seed=77, dtype=dtype)
    mask = c["mask"]
    nnz = int(mask.sum())
    drop = 5
    cap = nnz - drop
    trunc = mask.copy()
    rr, cc = np.nonzero(mask)                         # row-major = list order
    trunc[rr[cap:], cc[cap:]] = 0
    X, Wu, Wd, dY = (dev(c[k], dtype) for k in ("X", "W_up", "W_down", "dY"))

    def run(m, nnz_cap):
        bl = lx.lx_mask_compact(torch.from_numpy(m).cuda(), nnz_cap=nnz_cap)
        H = torch.full((nnz_cap * tile * tile + 4096,), float("nan"), dtype=X.dtype, device="cuda")
        Y = torch.full_like(X, float("nan"))
        lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, tile, tile, Y, H)
        assert torch.isnan(H[nnz_cap * tile * tile:]).all(), "wrote past the H_act buffer"
        dtc = lx_dtype(lx, dtype)
        ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(dtc, c["T"], c["d"], c["F"], tile,
                                                              tile, nnz_cap, 0) + 256,
                         dtype=torch.uint8, device="cuda")
        dX = torch.full_like(X, float("nan"))
        lx.lx_sparse_ffn_bwd_dx(dY, H, Wu, Wd, bl, tile, tile, dX, ws)
        torch.cuda.synchronize()
        return host(Y), host(dX), host(H[:nnz_cap * tile * tile])

    a = run(mask, cap)        # true list longer than the capacity
    b = run(trunc, cap)       # the truncated mask, exactly at capacity
    for x, y in zip(a, b):
        assert np.isfinite(x).all()
        assert np.array_equal(x, y)


@pytest.mark.parametrize("Tt,G,tiles_per_wg", [(64, 64, 0), (128, 128, 0), (64, 16, 1), (64, 16, 2), (64, 16, 4)])
def test_capacity_a_quarter_of_the_list(lx, Tt, G, tiles_per_wg):
    """A capacity far below the list's length (a quarter of it), on enough tiles that the items
    within the capacity would be dealt to workgroups the grid never launches if the item search
    counted the entries beyond it: every call gives the bits of the truncated mask.  G list rows
    for Tt token tiles (G < Tt: rows shared by Tt / G tiles, run with 1, 2 and 4 tiles per
    workgroup)."""
    import torch
    T, d, F = Tt * 64, 128, 2048
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, 0.5, seed=78 + Tt + G, dtype="bf16", w_std=0.05)
    gt = Tt // G
    mask = np.ascontiguousarray(c["mask"][:G])
    nnz = int(mask.sum())
    cap = nnz // 4
    trunc = mask.copy()
    rr, cc = np.nonzero(mask)
    trunc[rr[cap:], cc[cap:]] = 0
    X, Wu, Wd, dY = (dev(c[k], "bf16") for k in ("X", "W_up", "W_down", "dY"))

    def run(m):
        bl = lx.lx_mask_compact(torch.from_numpy(m).cuda(), nnz_cap=cap)
        nb = cap * gt
        H = torch.full((nb * 4096 + 4096,), float("nan"), dtype=X.dtype, device="cuda")
        Y = torch.full_like(X, float("nan"))
        ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(lx.LX_BF16, T, d, F, 64, 64, nb, 0) + 256,
                         dtype=torch.uint8, device="cuda")
        dX = torch.full_like(X, float("nan"))
        lx.lx_ffn_set_token_tiles_per_workgroup(tiles_per_wg)
        try:
            lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, 64, 64, Y, H)
            assert torch.isnan(H[nb * 4096:]).all(), "wrote past the H_act buffer"
            lx.lx_sparse_ffn_bwd_dx(dY, H, Wu, Wd, bl, 64, 64, dX, ws)
            torch.cuda.synchronize()
        finally:
            lx.lx_ffn_set_token_tiles_per_workgroup(0)
        return host(Y), host(dX), host(H[:nb * 4096])

    a, b = run(mask), run(trunc)
    for name, x, y in zip(("Y", "dX", "H"), a, b):
        assert np.isfinite(x).all(), name        # every block within the capacity was written
        assert np.array_equal(x, y), name


def _grouped_compact(dense, rows_mask, gt, tt, bn):
    """Dense [T,F] -> compact blocks in the order of a list whose row r covers the gt token
    tiles of group r: [row r][entry k][tile within the group]."""
    G, Fb = rows_mask.shape
    v = dense.reshape(G, gt, tt, Fb, bn)
    out = []
    for r in range(G):
        for j in np.nonzero(rows_mask[r])[0]:
            for g in range(gt):
                out.append(v[r, g, :, j, :])
    return np.stack(out) if out else np.zeros((0, tt, bn), dtype=dense.dtype)


@pytest.mark.parametrize("dtype,tile,T,d,F,G,density,seed", [
    ("bf16", 64, 512, 256, 1024, 1, 0.3, 81),     # one list for all tokens (the paper's case)
    ("bf16", 64, 512, 192, 704, 2, 0.4, 82),      # two groups of four tiles
    ("bf16", 64, 256, 128, 512, 1, 1.0, 83),      # shared and dense
    ("bf16", 64, 256, 128, 256, 1, 0.0, 84),      # shared and empty
    ("f32", 32, 256, 96, 384, 1, 0.3, 85),
    ("f32", 64, 256, 128, 512, 2, 0.5, 86),
])
def test_list_rows_shared_by_groups_of_token_tiles(lx, oracle, dtype, tile, T, d, F, G, density,
                                                   seed):
    """A list with fewer rows than token tiles: row r is the list of the tiles of group r.  The
    oracle sees the same thing as a dense mask with repeated rows."""
    import torch
    c = inputs.ffn_bernoulli(T, d, F, tile, tile, density, seed, dtype=dtype, w_std=0.05)
    Tt, Fb = T // tile, F // tile
    gt = Tt // G
    rows_mask = np.ascontiguousarray(c["mask"][:G])             # G independent rows
    full = np.repeat(rows_mask, gt, axis=0)
    H, Y = oracle.ffn_fwd(c["X"], c["W_up"], c["W_down"], full, tile, tile)
    Hq = round_to(H, dtype)
    _, dX = oracle.ffn_bwd_dx(c["dY"], c["W_up"], c["W_down"], full, Hq > 0, tile, tile)

    X, Wu, Wd, dY = (dev(c[k], dtype) for k in ("X", "W_up", "W_down", "dY"))
    bl = lx.lx_mask_compact(torch.from_numpy(rows_mask).cuda())
    assert bl.rows == G
    nblocks = bl.nnz_cap * gt
    Hd = torch.full((nblocks * tile * tile + 4096,), float("nan"), dtype=X.dtype, device="cuda")
    Yd = torch.full_like(X, float("nan"))
    lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, tile, tile, Yd, Hd)
    assert torch.isnan(Hd[nblocks * tile * tile:]).all(), "wrote past the H_act buffer"
    nnz = int(rows_mask.sum()) * gt
    got_H = host(Hd[:nnz * tile * tile]).reshape(nnz, tile, tile)
    ref_H = _grouped_compact(H, rows_mask, gt, tile, tile)
    H_in = torch.zeros_like(Hd)
    H_in[:nnz * tile * tile] = dev(_grouped_compact(Hq, rows_mask, gt, tile, tile).reshape(-1), dtype)
    dtc = lx_dtype(lx, dtype)
    ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(dtc, T, d, F, tile, tile, nblocks, 0) + 256,
                     dtype=torch.uint8, device="cuda")
    dXd = torch.full_like(X, float("nan"))
    lx.lx_sparse_ffn_bwd_dx(dY, H_in, Wu, Wd, bl, tile, tile, dXd, ws)
    torch.cuda.synchronize()
    pairs = dict(Y=(host(Yd), Y), dX=(host(dXd), dX))
    if nnz:
        pairs["H"] = (got_H, ref_H)
    for k, (g, r) in pairs.items():
        assert np.isfinite(g).all(), k
        if not r.any():
            assert not g.any(), k
            continue
        assert rel_err_max(g, r) <= TOL[dtype], (k, rel_err_max(g, r))
        assert rel_err_fro(g, r) <= FRO[dtype], (k, rel_err_fro(g, r))
    # the same problem with one list row per tile gives the same bits
    bl_full = lx.lx_mask_compact(torch.from_numpy(np.ascontiguousarray(full)).cuda())
    Y2 = torch.full_like(X, float("nan"))
    H2 = torch.empty(max(bl_full.nnz_cap, 1) * tile * tile, dtype=X.dtype, device="cuda")
    lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl_full, tile, tile, Y2, H2)
    torch.cuda.synchronize()
    assert np.array_equal(host(Y2), host(Yd))


@pytest.mark.parametrize("rows,nnz,tiles", [
    (16, 16, 1),    # 4 groups of entries: XCD rectangles of 4 tiles x 2 groups
    (16, 13, 1),    # the same with a ragged last group
    (8, 29, 1),     # 8 groups: 4 tiles x 4 groups
    (24, 8, 1),     # 6 tiles x 1 group
    (40, 3, 1),     # one group: 5 tiles per XCD
    (9, 8, 1),      # no cut divides 9 tiles: list order
    (64, 16, 4),    # four tiles per workgroup: 16 tile groups x 4 groups of entries
    (32, 8, 2),
])
def test_one_list_for_all_tiles_item_grid(lx, oracle, rows, nnz, tiles):
    """One list row for all token tiles: the sdd kernels deal the regular (tile, group of four
    entries) grid to the XCDs in rectangles where a cut divides it.  Y and dX equal, bit for bit,
    those of the same problem given as one list row per tile (items in list order); the first
    case is also checked against the oracle."""
    import torch
    T, d, Fb = rows * 64, 128, 32
    F = Fb * 64
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, 0.5, 900 + rows + nnz, dtype="bf16", w_std=0.05)
    row = np.zeros((1, Fb), np.uint8)
    row[0, np.random.default_rng(nnz).choice(Fb, nnz, replace=False)] = 1
    full = np.repeat(row, rows, axis=0)
    X, Wu, Wd, dY = (dev(c[k], "bf16") for k in ("X", "W_up", "W_down", "dY"))

    def run(mask, tiles_per_wg):
        bl = lx.lx_mask_compact(torch.from_numpy(np.ascontiguousarray(mask)).cuda())
        nblocks = bl.nnz_cap * (rows // mask.shape[0])
        ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(lx.LX_BF16, T, d, F, 64, 64, nblocks, 0) + 256,
                         dtype=torch.uint8, device="cuda")
        lx.lx_ffn_set_token_tiles_per_workgroup(tiles_per_wg)
        try:
            Hd = torch.zeros((nblocks * 4096,), dtype=X.dtype, device="cuda")
            Yd = torch.full_like(X, float("nan"))
            lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, 64, 64, Yd, Hd)
            dXd = torch.full_like(X, float("nan"))
            lx.lx_sparse_ffn_bwd_dx(dY, Hd, Wu, Wd, bl, 64, 64, dXd, ws)
            torch.cuda.synchronize()
        finally:
            lx.lx_ffn_set_token_tiles_per_workgroup(0)
        return host(Yd), host(dXd)

    Ys, dXs = run(row, tiles)
    Yt, dXt = run(full, 1)
    assert np.isfinite(Ys).all() and np.isfinite(dXs).all()
    assert np.array_equal(Ys, Yt) and np.array_equal(dXs, dXt)
    if (rows, nnz) == (16, 16):
        H, Y = oracle.ffn_fwd(c["X"], c["W_up"], c["W_down"], full, 64, 64)
        _, dX = oracle.ffn_bwd_dx(c["dY"], c["W_up"], c["W_down"], full, round_to(H, "bf16") > 0, 64, 64)
        for g, r in ((Ys, Y), (dXs, dX)):
            assert rel_err_max(g, r) <= TOL["bf16"] and rel_err_fro(g, r) <= FRO["bf16"]


@pytest.mark.parametrize("dtype,T,d,F,G,density,seed,bias", [
    ("bf16", 512, 192, 704, 2, 0.45, 181, False),   # two list rows, four tiles each; 11 blocks: ragged chunks of four
    ("bf16", 256, 128, 512, 1, 1.0, 182, True),     # one list for all tokens, dense, biases
    ("f16", 384, 320, 320, 3, 0.3, 183, False),     # three rows of two tiles; d not a multiple of 256
    ("bf16", 256, 128, 256, 1, 0.0, 184, False),    # empty list
    ("bf16", 1024, 128, 2048, 2, 0.2, 185, False),  # several workgroups per XCD range
])
def test_several_token_tiles_per_workgroup(lx, oracle, dtype, T, d, F, G, density, seed, bias):
    """Lists shared by an even number of tiles, run with two and with four token tiles per
    workgroup (the tuning knob): the results match the oracle and equal, bit for bit, those of
    the one-tile kernels -- every output element sees the same products in the same order."""
    import torch
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, density, seed, dtype=dtype, w_std=0.05)
    Tt = T // 64
    gt = Tt // G
    assert gt % 2 == 0
    rows_mask = np.ascontiguousarray(c["mask"][:G])
    full = np.repeat(rows_mask, gt, axis=0)
    rng = np.random.default_rng(seed)
    b_up = round_to(rng.standard_normal(F) * 0.1, dtype) if bias else None
    b_down = round_to(rng.standard_normal(d), dtype) if bias else None
    H, Y = oracle.ffn_fwd(c["X"], c["W_up"], c["W_down"], full, 64, 64, b_up, b_down)
    Hq = round_to(H, dtype)
    _, dX = oracle.ffn_bwd_dx(c["dY"], c["W_up"], c["W_down"], full, Hq > 0, 64, 64)

    X, Wu, Wd, dY = (dev(c[k], dtype) for k in ("X", "W_up", "W_down", "dY"))
    bu = dev(b_up, dtype) if bias else None
    bd = dev(b_down, dtype) if bias else None
    bl = lx.lx_mask_compact(torch.from_numpy(rows_mask).cuda())
    nblocks = max(bl.nnz_cap * gt, 1)
    nnz = int(rows_mask.sum()) * gt
    Wut, Wdt = lx.lx_ffn_pack_weights(Wu, Wd)
    ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(lx_dtype(lx, dtype), T, d, F, 64, 64, nblocks, 1)
                     + 256, dtype=torch.uint8, device="cuda")
    H_in = torch.zeros((nblocks * 4096,), dtype=X.dtype, device="cuda")
    H_in[:nnz * 4096] = dev(_grouped_compact(Hq, rows_mask, gt, 64, 64).reshape(-1), dtype)

    def run(tiles):
        lx.lx_ffn_set_token_tiles_per_workgroup(tiles)
        try:
            Hd = torch.full((nblocks * 4096 + 4096,), float("nan"), dtype=X.dtype, device="cuda")
            Yd = torch.full_like(X, float("nan"))
            lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, 64, 64, Yd, Hd, b_up=bu, b_down=bd)
            assert torch.isnan(Hd[nblocks * 4096:]).all(), "wrote past the H_act buffer"
            dXd = torch.full_like(X, float("nan"))
            lx.lx_sparse_ffn_bwd_dx(dY, H_in, Wu, Wd, bl, 64, 64, dXd, ws, W_up_t=Wut, W_down_t=Wdt)
            torch.cuda.synchronize()
        finally:
            lx.lx_ffn_set_token_tiles_per_workgroup(0)
        return host(Yd), host(Hd[:nnz * 4096]).reshape(nnz, 64, 64), host(dXd)

    four, two, one = run(4), run(2), run(1)     # (4 falls back to 2 where gt is not a multiple of 4)
    for multi in (four, two):
        for name, a, b in zip(("Y", "H", "dX"), multi, one):
            assert np.isfinite(a).all(), name
            assert np.array_equal(a, b), name
    refs = dict(Y=Y, H=_grouped_compact(H, rows_mask, gt, 64, 64), dX=dX)
    for name, g in zip(("Y", "H", "dX"), two):
        r = refs[name]
        if not r.any():
            assert not g.any(), name
            continue
        assert rel_err_max(g, r) <= TOL[dtype], (name, rel_err_max(g, r))
        assert rel_err_fro(g, r) <= FRO[dtype], (name, rel_err_fro(g, r))


def test_several_token_tiles_dsd_round_split(lx, oracle):
    """A shape whose four-tile dsd launch is whole rounds of workgroups plus a small rest
    (3 column chunks x 90 tile groups = 270 for 256 CUs): the rest, 20 tiles, goes to the two-tile kernel.
    The results equal those of one tile per workgroup bit for bit, and sampled tiles of both
    regions match the oracle."""
    import torch
    T, d, F = 360 * 64, 768, 256
    c = inputs.ffn_bernoulli(T, d, F, 64, 64, 0.75, 191, dtype="bf16", w_std=0.05)
    row = np.ascontiguousarray(c["mask"][:1])
    row[0, 0] = 1
    X, Wu, Wd, dY = (dev(c[k], "bf16") for k in ("X", "W_up", "W_down", "dY"))
    bl = lx.lx_mask_compact(torch.from_numpy(row).cuda())
    gt, nnz = T // 64, int(row.sum())
    nblocks = bl.nnz_cap * gt
    Wut, Wdt = lx.lx_ffn_pack_weights(Wu, Wd)
    ws = torch.empty(lx.lx_sparse_ffn_bwd_workspace_bytes(lx.LX_BF16, T, d, F, 64, 64, nblocks, 1) + 256,
                     dtype=torch.uint8, device="cuda")

    def run(tiles):
        lx.lx_ffn_set_token_tiles_per_workgroup(tiles)
        try:
            Hd = torch.zeros((nblocks * 4096,), dtype=X.dtype, device="cuda")
            Yd = torch.full_like(X, float("nan"))
            lx.lx_sparse_ffn_fwd(X, Wu, Wd, bl, 64, 64, Yd, Hd)
            dXd = torch.full_like(X, float("nan"))
            lx.lx_sparse_ffn_bwd_dx(dY, Hd, Wu, Wd, bl, 64, 64, dXd, ws, W_up_t=Wut, W_down_t=Wdt)
            torch.cuda.synchronize()
        finally:
            lx.lx_ffn_set_token_tiles_per_workgroup(0)
        return host(Yd), host(dXd)

    (Y4, dX4), (Y1, dX1) = run(4), run(1)
    assert np.isfinite(Y4).all() and np.isfinite(dX4).all()
    assert np.array_equal(Y4, Y1) and np.array_equal(dX4, dX1)
    for i in (3, 355):                        # a tile of the four-tile launch, one of the remainder
        sl = slice(i * 64, (i + 1) * 64)
        H, Y = oracle.ffn_fwd(c["X"][sl], c["W_up"], c["W_down"], row, 64, 64)
        assert rel_err_max(Y4[sl], Y) <= TOL["bf16"] and rel_err_fro(Y4[sl], Y) <= FRO["bf16"]
