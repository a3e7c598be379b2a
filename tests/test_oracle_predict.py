"""Pins of the oracle's MLP predictor (Sec. V-A, MLP block): approximate block
scores S = X Wa, threshold, OR-reduction over the tokens of a group.  CPU only."""
import numpy as np
import pytest


def _data(T, d, nblk, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, d)).astype(np.float32),
            (rng.standard_normal((d, nblk)) / np.sqrt(d)).astype(np.float32))


def test_brute_force_tiny(oracle):
    X, Wa = _data(6, 5, 4, 1)
    thr = 0.2
    S, M = oracle.mlp_predict(X, Wa, thr, group_rows=3)
    for t in range(6):
        for j in range(4):
            s = 0.0
            for k in range(5):
                s += float(X[t, k]) * float(Wa[k, j])
            assert abs(S[t, j] - s) < 1e-12
    for g in range(2):
        for j in range(4):
            want = any(S[t, j] > thr for t in range(3 * g, 3 * g + 3))
            assert M[g, j] == int(want)


def test_hand_example(oracle):
    # two tokens, two channels, two blocks: S = [[1*2 + 0*1, 1*(-1) + 0*3], [0.5*2 + 2*1, -0.5 + 6]]
    X = np.array([[1.0, 0.0], [0.5, 2.0]], dtype=np.float32)
    Wa = np.array([[2.0, -1.0], [1.0, 3.0]], dtype=np.float32)
    S, M = oracle.mlp_predict(X, Wa, 2.5)
    assert np.array_equal(S, np.array([[2.0, -1.0], [3.0, 5.5]]))
    assert np.array_equal(M, np.array([[1, 1]], dtype=np.uint8))
    _, M1 = oracle.mlp_predict(X, Wa, 2.5, group_rows=1)
    assert np.array_equal(M1, np.array([[0, 0], [1, 1]], dtype=np.uint8))
    _, M2 = oracle.mlp_predict(X, Wa, 3.0)             # strict comparison: 3.0 > 3.0 is false
    assert np.array_equal(M2, np.array([[0, 1]], dtype=np.uint8))


@pytest.mark.parametrize("group", [1, 8, 64, None])
def test_scores_are_a_matmul_and_reduction_is_max(oracle, group):
    """S equals the library product; OR over tokens of (S > thr) equals (max over tokens) > thr."""
    T, d, nblk = 64, 48, 24
    X, Wa = _data(T, d, nblk, 2)
    thr = {1: 0.8, 8: 1.5}.get(group, 2.3)         # keeps the mask away from all-ones
    S, M = oracle.mlp_predict(X, Wa, thr, group_rows=group)
    assert np.allclose(S, X.astype(np.float64) @ Wa.astype(np.float64), rtol=0, atol=1e-12)
    g = T if group is None else group
    want = (S.reshape(T // g, g, nblk).max(axis=1) > thr).astype(np.uint8)
    assert np.array_equal(M, want)
    assert 0 < M.mean() < 1                        # the case is not degenerate


def test_threshold_limits_and_monotonicity(oracle):
    X, Wa = _data(32, 16, 12, 3)
    _, lo = oracle.mlp_predict(X, Wa, -np.inf)
    _, hi = oracle.mlp_predict(X, Wa, np.inf)
    assert lo.all() and not hi.any()
    prev = None
    for thr in (-1.0, 0.0, 0.5, 1.0, 2.0):
        _, M = oracle.mlp_predict(X, Wa, thr, group_rows=8)
        if prev is not None:
            assert np.all(M <= prev)                # a higher threshold never adds a block
        prev = M


def test_coarser_groups_are_the_or_of_finer_ones(oracle):
    X, Wa = _data(64, 16, 10, 4)
    _, fine = oracle.mlp_predict(X, Wa, 0.6, group_rows=8)
    _, coarse = oracle.mlp_predict(X, Wa, 0.6, group_rows=32)
    assert np.array_equal(coarse, fine.reshape(2, 4, 10).max(axis=1))
