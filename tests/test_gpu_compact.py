"""GPU parity: mask compaction is bit-exact against the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lx():
    import torch
    assert torch.cuda.is_available()
    from paper_2510_15964_amd import lx
    return lx


def _check(lx, oracle, mask, transpose=False, offset=0):
    import torch
    if offset:   # the same bytes at an address that is `offset` past an aligned one
        buf = torch.empty(mask.size + offset, dtype=torch.uint8, device="cuda")
        m = buf[offset:].view(mask.shape)
        m.copy_(torch.from_numpy(mask))
        assert m.data_ptr() % 16 == offset % 16
    else:
        m = torch.from_numpy(mask).cuda()
    bl = lx.lx_mask_compact(m, transpose=transpose)
    torch.cuda.synchronize()
    flat = mask.reshape(-1, mask.shape[-2], mask.shape[-1])
    rps, cis, off = [np.zeros(1, np.int32)], [], 0
    for g in range(flat.shape[0]):
        rp, ci = oracle.mask_compact(flat[g], transpose=transpose)
        rps.append(rp[1:] + off)
        cis.append(ci)
        off += rp[-1]
    rp = np.concatenate(rps).astype(np.int32)
    ci = np.concatenate(cis).astype(np.int32) if cis else np.zeros(0, np.int32)
    got_rp = bl.row_ptr.cpu().numpy()
    assert np.array_equal(got_rp, rp)
    assert np.array_equal(bl.col_idx.cpu().numpy()[:rp[-1]], ci)


@pytest.mark.parametrize("shape,density", [
    ((16, 96), 0.3), ((64, 128), 0.11), ((128, 256), 0.08), ((64, 320), 0.05), ((64, 320), 1.0),
    ((1, 1), 1.0), ((1, 1), 0.0), ((3, 65), 0.5), ((7, 63), 0.5), ((5, 200), 0.0),
    ((32, 16, 16), 0.3), ((2, 32, 32, 32), 0.25), ((40, 32, 32), 0.5),
    ((9000, 5), 0.4),       # more rows than one scan pass holds
    ((4, 1100, 3), 0.7),
    ((3, 40000), 0.01),     # a row longer than the LDS staging buffer
])
@pytest.mark.parametrize("transpose", [False, True])
def test_compact_bit_exact(lx, oracle, shape, density, transpose):
    rng = np.random.default_rng(abs(hash((shape, density))) % (2 ** 31))
    mask = (rng.random(shape) < density).astype(np.uint8)
    mask[mask > 0] = rng.integers(1, 256, size=int(mask.sum()), dtype=np.uint8)
    _check(lx, oracle, mask, transpose)


@pytest.mark.parametrize("shape", [(7, 24, 40), (40, 32, 32), (33, 16, 16), (5, 61, 67)])
@pytest.mark.parametrize("offset", [1, 5, 15, 16])
@pytest.mark.parametrize("transpose", [False, True])
def test_compact_masks_at_any_address_and_parts_inside_a_mask(lx, oracle, shape, offset, transpose):
    """Masks large enough to be divided among workgroups: the rows before a part are counted
    16 bytes per load where whole masks precede it (at any alignment of the mask's address) and
    byte by byte inside the mask the part starts in."""
    rng = np.random.default_rng(1000 * offset + shape[0])
    mask = (rng.random(shape) < 0.4).astype(np.uint8)
    mask[mask > 0] = rng.integers(1, 256, size=int(mask.sum()), dtype=np.uint8)
    _check(lx, oracle, mask, transpose, offset)


def test_capacity_smaller_than_count_keeps_row_ptr_exact(lx, oracle):
    import torch
    rng = np.random.default_rng(5)
    mask = (rng.random((8, 40)) < 0.5).astype(np.uint8)
    m = torch.from_numpy(mask).cuda()
    guard = 64
    row_ptr = torch.empty(9, dtype=torch.int32, device="cuda")
    col = torch.full((10 + guard,), -7, dtype=torch.int32, device="cuda")
    bl = lx.BlockList(8, 40, row_ptr, col, 10)
    lx.lx_mask_compact(m, nnz_cap=10, out=bl)
    torch.cuda.synchronize()
    rp, ci = oracle.mask_compact(mask)
    assert np.array_equal(row_ptr.cpu().numpy(), rp)
    c = col.cpu().numpy()
    assert np.array_equal(c[:10], ci[:10]) and np.all(c[10:] == -7)


def test_pair_matches_single_lists(lx, oracle):
    import torch
    rng = np.random.default_rng(9)
    mask = (rng.random((2, 5, 24, 24)) < 0.35).astype(np.uint8)
    m = torch.from_numpy(mask).cuda()
    blr, blc = lx.lx_mask_compact_pair(m)
    a = lx.lx_mask_compact(m)
    b = lx.lx_mask_compact(m, transpose=True)
    torch.cuda.synchronize()
    nnz = int(mask.sum())
    for x, y in ((blr, a), (blc, b)):
        assert torch.equal(x.row_ptr, y.row_ptr) and torch.equal(x.col_idx[:nnz], y.col_idx[:nnz])
    rp, ci = oracle.mask_compact(mask[1, 3], transpose=True)
    r0 = (1 * 5 + 3) * 24
    got_rp = blc.row_ptr.cpu().numpy()[r0:r0 + 25]
    assert np.array_equal(got_rp - got_rp[0], rp)
    assert np.array_equal(blc.col_idx.cpu().numpy()[got_rp[0]:got_rp[-1]], ci)


def test_batch_matches_single_lists(lx, oracle):
    import torch
    rng = np.random.default_rng(10)
    m1 = (rng.random((64, 128)) < 0.1).astype(np.uint8)
    m2 = (rng.random((3, 16, 16)) < 0.4).astype(np.uint8)
    t1, t2 = torch.from_numpy(m1).cuda(), torch.from_numpy(m2).cuda()
    ref = [lx.lx_mask_compact(t1), lx.lx_mask_compact(t2), lx.lx_mask_compact(t2, transpose=True)]
    mk = lambda r: lx.BlockList(r.rows, r.cols, torch.zeros_like(r.row_ptr),
                                torch.zeros_like(r.col_idx), r.nnz_cap)
    outs = [mk(r) for r in ref]
    cb = lx.CompactBatch().add(t1, outs[0]).add(t2, outs[1]).add(t2, outs[2], transpose=True)
    lx.lx_mask_compact_batch(cb)
    torch.cuda.synchronize()
    for o, r, m in zip(outs, ref, (m1, m2, m2)):
        nnz = int(m.sum())
        assert torch.equal(o.row_ptr, r.row_ptr) and torch.equal(o.col_idx[:nnz], r.col_idx[:nnz])
    rp, ci = oracle.mask_compact(m1)
    assert np.array_equal(outs[0].row_ptr.cpu().numpy(), rp)
    assert np.array_equal(outs[0].col_idx.cpu().numpy()[:rp[-1]], ci)
