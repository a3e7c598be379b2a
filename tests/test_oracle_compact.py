"""Pins for the oracle's active-block list (Sec. VI-A / VI-B index lists)."""
import numpy as np
import pytest


@pytest.mark.parametrize("shape,density,seed", [((1, 1), 1.0, 0), ((16, 96), 0.3, 1),
                                               ((64, 128), 0.1, 2), ((7, 130), 0.5, 3),
                                               ((5, 9), 0.0, 4), ((3, 70), 1.0, 5)])
def test_scatter_back_and_popcount(oracle, shape, density, seed):
    rng = np.random.default_rng(seed)
    mask = (rng.random(shape) < density).astype(np.uint8)
    # non-{0,1} bytes count as set
    mask[mask > 0] = rng.integers(1, 255, size=int(mask.sum()), dtype=np.uint8)
    row_ptr, col_idx = oracle.mask_compact(mask)
    assert row_ptr[0] == 0 and row_ptr[-1] == np.count_nonzero(mask)
    assert np.all(np.diff(row_ptr) == np.count_nonzero(mask, axis=1))
    back = np.zeros(shape, dtype=bool)
    for r in range(shape[0]):
        cols = col_idx[row_ptr[r]:row_ptr[r + 1]]
        assert np.all(np.diff(cols) > 0), "ascending, no duplicates"
        back[r, cols] = True
    assert np.array_equal(back, mask != 0)


def test_matches_numpy_nonzero(oracle):
    rng = np.random.default_rng(11)
    mask = (rng.random((33, 77)) < 0.25).astype(np.uint8)
    row_ptr, col_idx = oracle.mask_compact(mask)
    r, c = np.nonzero(mask)           # row-major order == CSR order
    assert np.array_equal(col_idx, c.astype(np.int32))
    assert np.array_equal(row_ptr[1:], np.cumsum(np.bincount(r, minlength=33)))


def test_column_compressed_is_transpose(oracle):
    rng = np.random.default_rng(12)
    mask = (rng.random((20, 31)) < 0.4).astype(np.uint8)
    rp_t, ci_t = oracle.mask_compact(mask, transpose=True)
    rp, ci = oracle.mask_compact(np.ascontiguousarray(mask.T))
    assert np.array_equal(rp_t, rp) and np.array_equal(ci_t, ci)


def test_hand_example(oracle):
    mask = np.array([[0, 1, 1, 0], [0, 0, 0, 0], [1, 0, 0, 1]], dtype=np.uint8)
    rp, ci = oracle.mask_compact(mask)
    assert rp.tolist() == [0, 2, 2, 4]
    assert ci.tolist() == [1, 2, 0, 3]
