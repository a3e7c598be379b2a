"""Pins for the oracle's block-masked attention (Sec. IV-B mask semantics,
Sec. VI-A SDD -> softmax -> DSD, Sec. V-C backward mirrors forward)."""
import math

import numpy as np
import pytest
import torch

from paper_2510_15964_amd import inputs


def _case(seed, B=2, Hh=3, S=32, D=8, blk=8, density=0.5, causal=True,
          head_keep=1.0, mask_batch=1, force_diagonal=False):
    return inputs.attn_blocks(B, Hh, S, D, density, seed, dtype="f32", causal=causal,
                              head_keep=head_keep, blk=blk, mask_batch=mask_batch,
                              force_diagonal=force_diagonal)


def _allowed(c):
    """[mb,Hh,S,S] boolean element mask, no block logic downstream."""
    blk, S = c["blk"], c["S"]
    el = np.kron(c["mask"], np.ones((blk, blk))).astype(bool)
    if c["causal"]:
        el &= np.tril(np.ones((S, S), dtype=bool))
    el = el & (c["head_active"].astype(bool)[None, :, None, None])
    return el


def _torch_reference(c):
    """Element-wise masked softmax attention + autograd, fp64."""
    al = torch.tensor(np.broadcast_to(_allowed(c), (c["B"],) + _allowed(c).shape[1:]).copy())
    Q, K, V = (torch.tensor(c[k], dtype=torch.float64, requires_grad=True) for k in "QKV")
    s = c["scale"] * Q @ K.transpose(-1, -2)
    s = s.masked_fill(~al, float("-inf"))
    m = s.max(dim=-1, keepdim=True).values
    m = torch.where(torch.isinf(m), torch.zeros_like(m), m)
    e = torch.exp(s - m)
    l = e.sum(-1, keepdim=True)
    P = torch.where(l > 0, e / torch.where(l > 0, l, torch.ones_like(l)), torch.zeros_like(e))
    O = P @ V
    lse = torch.where(l > 0, m + torch.log(torch.where(l > 0, l, torch.ones_like(l))),
                      torch.full_like(l, float("-inf")))[..., 0]
    O.backward(torch.tensor(c["dO"], dtype=torch.float64))
    return (O.detach().numpy(), lse.detach().numpy(), Q.grad.numpy(), K.grad.numpy(),
            V.grad.numpy())


def _run(oracle, c):
    O, L = oracle.attn_fwd(c["Q"], c["K"], c["V"], c["mask"], c["scale"], c["causal"],
                           c["head_active"], c["blk"])
    dQ, dK, dV = oracle.attn_bwd(c["Q"], c["K"], c["V"], c["dO"], c["mask"], c["scale"],
                                 c["causal"], c["head_active"], c["blk"])
    return O, L, dQ, dK, dV


def test_hand_example(oracle):
    """Two tokens, one channel, causal.  Row 0 sees key 0 only: O = V0 = 1,
    LSE = q0 k0 = 1.  Row 1: scores (2, 6), O = (e^2 - e^6)/(e^2 + e^6) =
    -tanh(2), LSE = 6 + log(1 + e^-4)."""
    Q = np.array([[[[1.0], [2.0]]]], dtype=np.float32)
    K = np.array([[[[1.0], [3.0]]]], dtype=np.float32)
    V = np.array([[[[1.0], [-1.0]]]], dtype=np.float32)
    mask = np.ones((1, 1, 2, 2), dtype=np.uint8)
    O, L = oracle.attn_fwd(Q, K, V, mask, 1.0, 1, None, blk=1)
    assert O[0, 0, 0, 0] == 1.0 and L[0, 0, 0] == 1.0
    assert abs(O[0, 0, 1, 0] + math.tanh(2.0)) < 1e-15
    assert abs(L[0, 0, 1] - (6.0 + math.log1p(math.exp(-4.0)))) < 1e-15
    # dropping block (1,0): row 1 sees key 1 only -> O = V1
    mask[0, 0, 1, 0] = 0
    O, L = oracle.attn_fwd(Q, K, V, mask, 1.0, 1, None, blk=1)
    assert O[0, 0, 1, 0] == -1.0 and L[0, 0, 1] == 6.0


@pytest.mark.parametrize("causal", [True, False])
def test_all_ones_mask_is_library_attention(oracle, causal):
    c = _case(1, density=1.0, causal=causal)
    O, L, dQ, dK, dV = _run(oracle, c)
    Q, K, V = (torch.tensor(c[k], dtype=torch.float64, requires_grad=True) for k in "QKV")
    Ot = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=causal,
                                                          scale=c["scale"])
    Ot.backward(torch.tensor(c["dO"], dtype=torch.float64))
    np.testing.assert_allclose(O, Ot.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dQ, Q.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, K.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, V.grad.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("seed,kw", [
    (2, dict()), (3, dict(causal=False, density=0.3)),
    (4, dict(head_keep=0.5)), (5, dict(mask_batch=2, density=0.4)),
    (6, dict(force_diagonal=True, density=0.4)), (7, dict(B=1, Hh=2, S=48, D=5, blk=16)),
])
def test_elementwise_mask_and_autograd(oracle, seed, kw):
    c = _case(seed, **kw)
    got = _run(oracle, c)
    ref = _torch_reference(c)
    for g, r, name in zip(got, ref, "O LSE dQ dK dV".split()):
        assert np.array_equal(np.isneginf(g), np.isneginf(r)), name
        fin = np.isfinite(r)
        np.testing.assert_allclose(g[fin], r[fin], rtol=1e-10, atol=1e-12, err_msg=name)


def test_empty_mask_and_inactive_heads_give_zero(oracle):
    c = _case(8)
    c["mask"][:] = 0
    O, L, dQ, dK, dV = _run(oracle, c)
    assert not O.any() and not dQ.any() and not dK.any() and not dV.any()
    assert np.all(np.isneginf(L))
    c = _case(9, density=1.0)
    c["head_active"][:] = [1, 0, 1]
    O, L, dQ, dK, dV = _run(oracle, c)
    for a in (O, dQ, dK, dV):
        assert not a[:, 1].any() and a[:, 0].any() and a[:, 2].any()
    assert np.all(np.isneginf(L[:, 1])) and np.all(np.isfinite(L[:, 0]))


def test_rows_without_allowed_key(oracle):
    """Literal Bernoulli masks leave early query blocks without any key."""
    c = _case(10, density=0.3)
    c["mask"][:, :, 0, :] = 0
    O, L, dQ, dK, dV = _run(oracle, c)
    blk = c["blk"]
    assert not O[:, :, :blk].any() and np.all(np.isneginf(L[:, :, :blk]))
    assert not dQ[:, :, :blk].any()
    assert all(np.isfinite(a).all() for a in (O, dQ, dK, dV))


def test_closed_forms(oracle):
    c = _case(11, density=0.5, force_diagonal=True)
    al = np.broadcast_to(_allowed(c), (c["B"],) + _allowed(c).shape[1:])
    # Q = 0: uniform attention -> O = mean of V over the allowed keys, LSE = log(count)
    c0 = dict(c)
    c0["Q"] = np.zeros_like(c["Q"])
    O, L = oracle.attn_fwd(c0["Q"], c["K"], c["V"], c["mask"], c["scale"], 1, None, c["blk"])
    cnt = al.sum(-1)
    mean = (al[..., None] * c["V"].astype(np.float64)[:, :, None, :, :]).sum(-2) / cnt[..., None]
    np.testing.assert_allclose(O, mean, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(L, np.log(cnt), rtol=1e-12, atol=1e-13)
    # V = 1: rows of P sum to one -> O = 1; dS rows sum to zero, so with K = 1: dQ = 0
    ones = np.ones_like(c["V"])
    O, _ = oracle.attn_fwd(c["Q"], c["K"], ones, c["mask"], c["scale"], 1, None, c["blk"])
    np.testing.assert_allclose(O, 1.0, rtol=0, atol=1e-13)
    dQ, dK, dV = oracle.attn_bwd(c["Q"], ones, c["V"], c["dO"], c["mask"], c["scale"], 1, None,
                                 c["blk"])
    np.testing.assert_allclose(dQ, 0.0, atol=1e-12)
    # softmax is invariant to a shift of all scores of a row: K -> K + a*1 adds
    # a*sum(Q[q]) to every score of row q and must not change O
    Kshift = (c["K"] + np.float32(0.5))
    O1, _ = oracle.attn_fwd(c["Q"], c["K"], c["V"], c["mask"], c["scale"], 1, None, c["blk"])
    O2, _ = oracle.attn_fwd(c["Q"], Kshift, c["V"], c["mask"], c["scale"], 1, None, c["blk"])
    # (K + 0.5 is rounded to fp32, so the shift is exact only to ~6e-8)
    np.testing.assert_allclose(O1, O2, rtol=0, atol=2e-6)


def test_backward_matches_finite_differences(oracle):
    c = _case(12, B=1, Hh=1, S=4, D=2, blk=2, density=1.0)
    c["mask"][0, 0] = [[1, 0], [1, 1]]
    O, L, dQ, dK, dV = _run(oracle, c)
    dO = c["dO"].astype(np.float64)
    eps = 2.0 ** -12

    def loss(Q, K, V):
        Op, _ = oracle.attn_fwd(Q, K, V, c["mask"], c["scale"], 1, None, 2)
        return (dO * Op).sum()

    for name, grad in (("Q", dQ), ("K", dK), ("V", dV)):
        for idx in np.ndindex(4, 2):
            vals = []
            for sgn in (+1, -1):
                t = {k: c[k].copy() for k in "QKV"}
                t[name][0, 0][idx] = np.float32(t[name][0, 0][idx] + sgn * eps)
                vals.append(loss(t["Q"], t["K"], t["V"]))
            fd = (vals[0] - vals[1]) / (2 * eps)
            assert abs(fd - grad[0, 0][idx]) < 5e-7 * max(1.0, abs(fd)), (name, idx)


def test_masked_blocks_are_never_read(oracle):
    """0 means non-computation: NaN in K / V blocks that no query block of a
    head uses must not reach any output."""
    c = _case(13, B=1, Hh=2, S=32, D=4, blk=8, density=0.5)
    c["mask"][0, :, :, 2] = 0          # key block 2 unused by every query block
    ref = _run(oracle, c)
    K = c["K"].copy()
    V = c["V"].copy()
    K[:, :, 16:24] = np.nan
    V[:, :, 16:24] = np.nan
    c2 = dict(c, K=K, V=V)
    got = _run(oracle, c2)
    for g, r, name in zip(got, ref, "O LSE dQ dK dV".split()):
        assert np.array_equal(g, r), name


def test_config3_generator():
    c = inputs.attn_blocks(1, 32, 1024, 64, 0.30, 3000, head_keep=0.875)
    nb = 16
    causal_blocks = nb * (nb + 1) // 2
    dens = c["mask"].sum() / (32 * causal_blocks)
    assert 0.27 < dens < 0.33
    assert not np.triu(c["mask"][0, 0], 1).any()
    assert 20 <= c["head_active"].sum() <= 32
