"""Pins of the oracle's LoRA-branch FFN (Sec. II-C / II-D): z = W x + B A x under the block mask,
and the gradients of the input and of the trainable A, B."""
import numpy as np
import pytest


def _case(T, d, F, r, tile, seed, density=0.5):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    X, dY = f(T, d), f(T, d)
    Wu, Wd = f(F, d) / np.sqrt(d), f(d, F) / np.sqrt(F)
    A, B = f(r, d) / np.sqrt(d), f(F, r) * 0.3
    mask = (rng.random((T // tile, F // tile)) < density).astype(np.uint8)
    return X, dY, Wu.astype(np.float32), Wd.astype(np.float32), A.astype(np.float32), B.astype(np.float32), mask


def _dense(mask, tile):
    return np.kron(mask, np.ones((tile, tile), dtype=np.uint8)).astype(bool)


def test_forward_is_the_plain_ffn_with_merged_weights(oracle):
    """z = (W + B A) x: the LoRA forward equals the plain masked FFN on W + B A (Sec. II-D)."""
    X, dY, Wu, Wd, A, B, mask = _case(64, 24, 96, 5, 32, 1)
    U, H, Y = oracle.ffn_lora_fwd(X, Wu, A, B, Wd, mask, 32, 32)
    merged = (Wu.astype(np.float64) + B.astype(np.float64) @ A.astype(np.float64))
    Z = X.astype(np.float64) @ merged.T
    Href = np.where(_dense(mask, 32), np.maximum(Z, 0), 0)
    assert np.allclose(U, X.astype(np.float64) @ A.astype(np.float64).T, rtol=1e-12, atol=1e-12)
    assert np.allclose(H, Href, rtol=1e-10, atol=1e-12)
    assert np.allclose(Y, Href @ Wd.astype(np.float64).T, rtol=1e-10, atol=1e-12)


def test_zero_branch_reduces_to_the_base_oracle(oracle):
    X, dY, Wu, Wd, A, B, mask = _case(64, 16, 64, 4, 32, 2)
    for A0, B0 in ((A, np.zeros_like(B)), (np.zeros_like(A), B)):
        U, H, Y = oracle.ffn_lora_fwd(X, Wu, A0, B0, Wd, mask, 32, 32)
        H0, Y0 = oracle.ffn_fwd(X, Wu, Wd, mask, 32, 32)
        assert np.array_equal(H, H0) and np.array_equal(Y, Y0)
        g = oracle.ffn_lora_bwd(X, dY, Wu, A0, B0, Wd, mask, H > 0, U, 32, 32)
        dZ0, dX0 = oracle.ffn_bwd_dx(dY, Wu, Wd, mask, H0 > 0, 32, 32)
        assert np.array_equal(g["dZ"], dZ0)
        if not B0.any():
            assert np.allclose(g["dX"], dX0, rtol=1e-12, atol=1e-12) and not g["dA"].any()


def test_gradients_match_autograd(oracle):
    """Library pin: torch autograd (fp64) through the dense masked formula."""
    import torch
    X, dY, Wu, Wd, A, B, mask = _case(96, 20, 64, 6, 32, 3, density=0.6)
    U, H, Y = oracle.ffn_lora_fwd(X, Wu, A, B, Wd, mask, 32, 32)
    g = oracle.ffn_lora_bwd(X, dY, Wu, A, B, Wd, mask, H > 0, U, 32, 32)
    t = lambda a, rg=False: torch.tensor(a, dtype=torch.float64, requires_grad=rg)
    Xt, At, Bt = t(X, True), t(A, True), t(B, True)
    Z = Xt @ t(Wu).T + (Xt @ At.T) @ Bt.T
    Ht = torch.relu(Z) * t(_dense(mask, 32).astype(np.float64))
    Yt = Ht @ t(Wd).T
    Yt.backward(t(dY))
    assert np.allclose(Y, Yt.detach().numpy(), rtol=1e-10, atol=1e-12)
    for name, ref in (("dX", Xt.grad), ("dA", At.grad), ("dB", Bt.grad)):
        assert np.allclose(g[name], ref.numpy(), rtol=1e-9, atol=1e-11), name


def test_inactive_blocks_get_no_gradient_and_are_never_read(oracle):
    """Rows of dB of a neuron block that no token tile lists are zero; poisoning the weights of
    inactive (tile, block) pairs changes nothing (Sec. II-D's conclusion)."""
    X, dY, Wu, Wd, A, B, mask = _case(64, 16, 128, 4, 32, 4, density=0.4)
    mask[:, 1] = 0
    U, H, Y = oracle.ffn_lora_fwd(X, Wu, A, B, Wd, mask, 32, 32)
    g = oracle.ffn_lora_bwd(X, dY, Wu, A, B, Wd, mask, H > 0, U, 32, 32)
    assert not g["dB"][32:64].any()
    Wu2, B2, Wd2 = Wu.copy(), B.copy(), Wd.copy()
    Wu2[32:64] = np.nan
    B2[32:64] = np.nan
    Wd2[:, 32:64] = np.nan
    U2, H2, Y2 = oracle.ffn_lora_fwd(X, Wu2, A, B2, Wd2, mask, 32, 32)
    assert np.array_equal(H, H2) and np.array_equal(Y, Y2)


def test_finite_differences_of_the_trainable_matrices(oracle):
    X, dY, Wu, Wd, A, B, mask = _case(32, 8, 32, 3, 32, 5, density=1.0)
    U, H, Y = oracle.ffn_lora_fwd(X, Wu, A, B, Wd, mask, 32, 32)
    g = oracle.ffn_lora_bwd(X, dY, Wu, A, B, Wd, mask, H > 0, U, 32, 32)
    loss = lambda A_, B_: float((oracle.ffn_lora_fwd(X, Wu, A_, B_, Wd, mask, 32, 32)[2] * dY).sum())
    eps = 1e-3
    for (q, k) in ((0, 0), (2, 5)):
        Ap, Am = A.copy(), A.copy()
        Ap[q, k] += eps
        Am[q, k] -= eps
        assert abs((loss(Ap, B) - loss(Am, B)) / (2 * eps) - g["dA"][q, k]) < 2e-3 * max(1, abs(g["dA"][q, k]))
    for (f, q) in ((1, 0), (17, 2)):
        Bp, Bm = B.copy(), B.copy()
        Bp[f, q] += eps
        Bm[f, q] -= eps
        assert abs((loss(A, Bp) - loss(A, Bm)) / (2 * eps) - g["dB"][f, q]) < 2e-3 * max(1, abs(g["dB"][f, q]))
