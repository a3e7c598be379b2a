"""Pins for the oracle's masked FFN (Sec. II-C, II-D, VI-B).

Every check compares the oracle with something that is not the oracle: a
library routine on the dense special case, an element-wise-mask formula with no
block logic, autograd, finite differences, hand-computed values, or an
invariant of the mathematics.
"""
import json
import os

import numpy as np
import pytest
import torch

from paper_2510_15964_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _small(seed, T=64, d=40, F=96, tile_t=16, blk_n=8, density=0.4, bias=False):
    c = inputs.ffn_bernoulli(T, d, F, tile_t, blk_n, density, seed, w_std=0.3)
    if bias:
        rng = np.random.default_rng(seed + 99)
        c["b_up"] = rng.standard_normal(F).astype(np.float32)
        c["b_down"] = rng.standard_normal(d).astype(np.float32)
    return c


def _elementwise_reference(c, mask=None):
    """Independent fp64 formulation: library matmuls and an element-wise mask."""
    mask = c["mask"] if mask is None else mask
    Mel = np.kron(mask, np.ones((c["tile_t"], c["blk_n"]))).astype(bool)
    X = c["X"].astype(np.float64)
    Wu = c["W_up"].astype(np.float64)
    Wd = c["W_down"].astype(np.float64)
    Z = X @ Wu.T + (c.get("b_up", 0.0))
    H = np.where(Mel & (Z > 0), Z, 0.0)
    Y = H @ Wd.T + (c.get("b_down", 0.0))
    dY = c["dY"].astype(np.float64)
    dH = dY @ Wd
    dZ = np.where(Mel & (Z > 0), dH, 0.0)
    dX = dZ @ Wu
    return H, Y, dZ, dX


def _run(oracle, c, mask=None):
    mask = c["mask"] if mask is None else mask
    H, Y = oracle.ffn_fwd(c["X"], c["W_up"], c["W_down"], mask, c["tile_t"],
                          c["blk_n"], c.get("b_up"), c.get("b_down"))
    dZ, dX = oracle.ffn_bwd_dx(c["dY"], c["W_up"], c["W_down"], mask, H > 0,
                               c["tile_t"], c["blk_n"])
    return H, Y, dZ, dX


def test_hand_example(oracle):
    g = json.load(open(os.path.join(GOLD, "ffn_hand.json")))
    a = lambda k: np.array(g[k], dtype=np.float32)
    mask = np.array(g["mask"], dtype=np.uint8)
    H, Y = oracle.ffn_fwd(a("X"), a("W_up"), a("W_down"), mask, 1, 1)
    dZ, dX = oracle.ffn_bwd_dx(a("dY"), a("W_up"), a("W_down"), mask, H > 0, 1, 1)
    assert np.array_equal(H, a("H")) and np.array_equal(Y, a("Y"))
    assert np.array_equal(dZ, a("dZ")) and np.array_equal(dX, a("dX"))


@pytest.mark.parametrize("bias", [False, True])
def test_all_ones_mask_is_the_dense_layer(oracle, bias):
    """Special case that reduces to library routines (torch fp64)."""
    c = _small(1, bias=bias)
    ones = np.ones_like(c["mask"])
    H, Y, dZ, dX = _run(oracle, c, ones)
    X = torch.tensor(c["X"], dtype=torch.float64, requires_grad=True)
    Wu = torch.tensor(c["W_up"], dtype=torch.float64)
    Wd = torch.tensor(c["W_down"], dtype=torch.float64)
    bu = torch.tensor(c["b_up"], dtype=torch.float64) if bias else None
    bd = torch.tensor(c["b_down"], dtype=torch.float64) if bias else None
    Ht = torch.relu(torch.nn.functional.linear(X, Wu, bu))
    Yt = torch.nn.functional.linear(Ht, Wd, bd)
    Yt.backward(torch.tensor(c["dY"], dtype=torch.float64))
    np.testing.assert_allclose(H, Ht.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Y, Yt.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX, X.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_empty_mask_is_zero(oracle):
    c = _small(2, bias=True)
    zero = np.zeros_like(c["mask"])
    H, Y, dZ, dX = _run(oracle, c, zero)
    assert not H.any() and not dZ.any() and not dX.any()
    assert np.array_equal(Y, np.broadcast_to(c["b_down"].astype(np.float64), Y.shape))
    del c["b_up"], c["b_down"]
    H, Y, dZ, dX = _run(oracle, c, zero)
    assert not Y.any()


@pytest.mark.parametrize("seed,bias", [(3, False), (4, True), (5, False)])
def test_elementwise_mask_brute_force(oracle, seed, bias):
    c = _small(seed, T=48, d=24, F=64, tile_t=8, blk_n=16, density=0.35, bias=bias)
    got = _run(oracle, c)
    ref = _elementwise_reference(c)
    for g, r, name in zip(got, ref, "H Y dZ dX".split()):
        np.testing.assert_allclose(g, r, rtol=1e-11, atol=1e-12, err_msg=name)


def test_backward_matches_autograd_of_elementwise_formula(oracle):
    c = _small(6, T=96, d=48, F=160, tile_t=32, blk_n=32, density=0.5)
    H, Y, dZ, dX = _run(oracle, c)
    Mel = torch.tensor(np.kron(c["mask"], np.ones((32, 32))), dtype=torch.float64)
    X = torch.tensor(c["X"], dtype=torch.float64, requires_grad=True)
    Wu = torch.tensor(c["W_up"], dtype=torch.float64)
    Wd = torch.tensor(c["W_down"], dtype=torch.float64)
    Yt = (torch.relu(X @ Wu.T) * Mel) @ Wd.T
    Yt.backward(torch.tensor(c["dY"], dtype=torch.float64))
    np.testing.assert_allclose(Y, Yt.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dX, X.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_backward_matches_finite_differences(oracle):
    """dX is the gradient of L = sum(dY * Y(X)); central differences in fp64
    on a tiny layer, away from ReLU kinks."""
    c = _small(7, T=4, d=3, F=4, tile_t=2, blk_n=2, density=0.6)
    c["mask"][:] = [[1, 0], [1, 1]]
    H, Y, dZ, dX = _run(oracle, c)
    assert np.abs(H[H != 0]).min() > 1e-2  # no pre-activation near the kink
    dY = c["dY"].astype(np.float64)
    eps = 2.0 ** -10   # exactly representable; X +- eps stays fp32-exact
    X0 = c["X"].copy()
    for t in range(4):
        for k in range(3):
            Ls = []
            for sgn in (+1, -1):
                Xp = X0.copy()
                Xp[t, k] = np.float32(Xp[t, k] + sgn * eps)
                assert float(Xp[t, k]) - float(X0[t, k]) == sgn * eps
                _, Yp = oracle.ffn_fwd(Xp, c["W_up"], c["W_down"], c["mask"], 2, 2)
                Ls.append((dY * Yp).sum())
            fd = (Ls[0] - Ls[1]) / (2 * eps)
            # the layer is piecewise linear: central differences are exact
            assert abs(fd - dX[t, k]) < 1e-9 * max(1.0, abs(fd))


def test_mask_equal_to_relu_support_is_bitwise_dense(oracle):
    """ReLU zeros are exact zeros (Sec. II-B): skipping a block whose
    activations are all zero changes nothing, bit for bit."""
    c = inputs.ffn_planted_support(256, 96, 512, 32, 32, 0.5, 4.0, seed=8, dtype="bf16")
    ones = np.ones_like(c["mask"])
    Hd, Yd, dZd, dXd = _run(oracle, c, ones)
    support = (Hd.reshape(8, 32, 16, 32) > 0).any(axis=(1, 3)).astype(np.uint8)
    assert np.array_equal(support, c["mask"]), "generator plants the true support"
    assert 0.02 < c["mask"].mean() < 0.5
    Hs, Ys, dZs, dXs = _run(oracle, c)
    for a, b in ((Hd, Hs), (Yd, Ys), (dZd, dZs), (dXd, dXs)):
        assert np.array_equal(a, b)


def test_positive_homogeneity_and_mask_additivity(oracle):
    c = _small(9)
    H, Y, dZ, dX = _run(oracle, c)
    c2 = dict(c)
    c2["X"] = c["X"] * np.float32(4.0)        # exact scaling in fp32
    H2, Y2, _, _ = _run(oracle, c2)
    np.testing.assert_allclose(Y2, 4.0 * Y, rtol=1e-13, atol=0)
    rng = np.random.default_rng(0)
    split = rng.random(c["mask"].shape) < 0.5
    m1 = (c["mask"] * split).astype(np.uint8)
    m2 = (c["mask"] * ~split).astype(np.uint8)
    _, Y_1, _, dX_1 = _run(oracle, c, m1)
    _, Y_2, _, dX_2 = _run(oracle, c, m2)
    np.testing.assert_allclose(Y_1 + Y_2, Y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dX_1 + dX_2, dX, rtol=1e-12, atol=1e-13)


def test_inactive_blocks_are_never_read(oracle):
    """Sec. II-D: parameters inactive in the forward pass are excluded from
    the backward pass too.  Poison them with NaN: nothing may change."""
    c = _small(10, T=32, d=24, F=64, tile_t=16, blk_n=8, density=0.4)
    ref = _run(oracle, c)
    for i in range(c["mask"].shape[0]):          # one token tile at a time
        sl = slice(i * 16, (i + 1) * 16)
        Wu = c["W_up"].copy()
        Wd = c["W_down"].copy()
        for j in np.nonzero(c["mask"][i] == 0)[0]:
            Wu[j * 8:(j + 1) * 8, :] = np.nan
            Wd[:, j * 8:(j + 1) * 8] = np.nan
        H, Y = oracle.ffn_fwd(c["X"][sl], Wu, Wd, c["mask"][i:i + 1], 16, 8)
        dZ, dX = oracle.ffn_bwd_dx(c["dY"][sl], Wu, Wd, c["mask"][i:i + 1],
                                   H > 0, 16, 8)
        for g, r in zip((H, Y, dZ, dX), ref):
            assert np.array_equal(g, r[sl])


def test_relu_derivative_is_zero_at_zero(oracle):
    """A pre-activation of exactly 0 passes no gradient (strict Z > 0)."""
    X = np.array([[1.0, -1.0]], dtype=np.float32)
    W_up = np.array([[1.0, 1.0], [2.0, 1.0]], dtype=np.float32)   # Z = [0, 1]
    W_down = np.array([[1.0, 1.0], [0.0, 0.0]], dtype=np.float32)
    mask = np.ones((1, 1), dtype=np.uint8)
    H, Y = oracle.ffn_fwd(X, W_up, W_down, mask, 1, 2)
    dY = np.array([[1.0, 0.0]], dtype=np.float32)
    dZ, dX = oracle.ffn_bwd_dx(dY, W_up, W_down, mask, H > 0, 1, 2)
    assert H.tolist() == [[0.0, 1.0]] and dZ.tolist() == [[0.0, 1.0]]
    assert dX.tolist() == [[2.0, 1.0]]


def test_config1_generator_shape_and_density():
    c = inputs.config1_ffn()
    assert c["X"].shape == (512, 768) and c["W_up"].shape == (3072, 768)
    assert c["mask"].shape == (16, 96) and 0.25 < c["mask"].mean() < 0.35
    assert abs(c["W_up"].std() - 0.02) < 1e-3
