"""The ideal 16-bit pipeline, emulated in fp64 (test infrastructure; imports neither the HIP binding
nor the oracle).

A 16-bit run of the operator cannot reproduce the fp64 oracle: whatever the kernel design, the
factor that feeds the second matrix product (H, dZ for the FFN; P, dS for attention) exists only as
a 16-bit value, and so does every output.  The functions here compute the operator in fp64 with
exactly those roundings and no other: one rounding of the intermediate factor, one of the output;
everything else (products, sums, softmax statistics) is exact to fp64.  The distance of their result
from the oracle's is the error no 16-bit implementation can avoid on that input, and it is what the
parity tests derive their element-wise gate from (tests/util.py: assert_within_emulated).

The figure is a maximum over 10^5 .. 10^6 rounding errors, so it depends on which values happen to
be rounded.  For attention a fused kernel is free in one respect that changes those values: the
reference point the unnormalised probabilities are taken against (any upper bound of the row's
scores gives the same softmax).  attn() therefore takes that reference point as a parameter and
attn_realisations() returns the pipeline for eight of them, spread over the one period (a factor
of two) after which the rounding repeats; between them the figure of one tensor varies by up to a
factor of two (test_emulated_gate.py), and the gate is taken from their envelope.

The roundings, per tensor:
  FFN        H = round(ReLU(X W_up^T + b));  Y = round(H W_down^T + b);
             dZ = round((dY W_down) (.) [H > 0]);  dX = round(dZ W_up)
  attention  P' = round(exp(S - m)) (unnormalised, as a fused kernel holds it), the row sum l of the
             unrounded exponentials;  O = round(P' V / l);
             Delta = rowsum(dO (.) O) from the stored (rounded) O;
             P = round(exp(S - LSE));  dS = round(P_exact (.) (dO V^T - Delta));
             dV = round(P^T dO);  dQ = round(scale dS K);  dK = round(scale dS^T Q)
"""
from __future__ import annotations

import numpy as np

from paper_2510_15964_amd.inputs import bf16_round, f16_round


def _r(a, dtype):
    a32 = np.asarray(a, dtype=np.float32)
    out = bf16_round(a32) if dtype == "bf16" else f16_round(a32) if dtype == "f16" else a32
    return out.astype(np.float64)


def ffn(c, mask=None, b_up=None, b_down=None, act=None):
    """Emulated Y, H, dX of FFN workload dict `c` (as paper_2510_15964_amd.inputs builds them) under
    block mask `mask` [T/tile, F/blk].  act: the activation map [T,F] the backward pass gates with
    (default: the emulated rounded H > 0)."""
    dt, tt, bn = c["dtype"], c["tile_t"], c["blk_n"]
    mask = c["mask"] if mask is None else mask
    X, Wu, Wd, dY = (np.asarray(c[k], np.float64) for k in ("X", "W_up", "W_down", "dY"))
    M = np.kron(mask.astype(bool), np.ones((tt, bn), dtype=bool))
    Z = X @ Wu.T
    if b_up is not None:
        Z = Z + np.asarray(b_up, np.float64)[None, :]
    H = _r(np.where(M, np.maximum(Z, 0.0), 0.0), dt)
    Y = H @ Wd.T
    if b_down is not None:
        Y = Y + np.asarray(b_down, np.float64)[None, :]
    A = (H > 0) if act is None else np.asarray(act, bool)
    dZ = _r(np.where(M & A, dY @ Wd, 0.0), dt)
    return dict(H=H, Y=_r(Y, dt), dX=_r(dZ @ Wu, dt))


def attn(c, ref_shift=0.0):
    """Emulated O, dQ, dK, dV of attention workload dict `c` (inputs.attn_blocks).
    ref_shift: the unnormalised probabilities are taken relative to the row maximum plus this
    offset (natural-log units) instead of the row maximum itself -- mathematically the same softmax
    (a fused kernel with a running maximum holds them relative to SOME upper bound of the row),
    but another realisation of the rounding of P'."""
    dt = c.get("dtype", "bf16")
    B, Hh, S, blk = c["B"], c["Hh"], c["S"], c["blk"]
    Q, K, V, dO = (np.asarray(c[k], np.float64) for k in ("Q", "K", "V", "dO"))
    mask = np.asarray(c["mask"], bool)
    if mask.ndim == 3:
        mask = mask[None]
    el = np.kron(mask, np.ones((blk, blk), dtype=bool))               # [mb, Hh, S, S]
    if c["causal"]:
        el = el & np.tril(np.ones((S, S), dtype=bool))
    ha = c.get("head_active")
    if ha is not None:
        el = el & np.asarray(ha, bool)[None, :, None, None]
    el = np.broadcast_to(el, (B, Hh, S, S))
    out = {k: np.zeros_like(Q) for k in ("O", "dQ", "dK", "dV")}
    scale = float(c["scale"])
    for b in range(B):
        for h in range(Hh):
            e = el[b, h]
            q, k, v, do = Q[b, h], K[b, h], V[b, h], dO[b, h]
            s = np.where(e, scale * (q @ k.T), -np.inf)
            m = s.max(-1, keepdims=True)
            m = np.where(np.isinf(m), 0.0, m)
            E = np.exp(s - m - ref_shift)
            l = E.sum(-1, keepdims=True)
            ok = l > 0
            ls = np.where(ok, l, 1.0)
            O = _r(np.where(ok, (_r(E, dt) @ v) / ls, 0.0), dt)
            P = np.where(e, E / ls, 0.0)                               # exp(S - LSE), exact
            delta = (do * O).sum(-1, keepdims=True)
            dS = _r(P * (do @ v.T - delta), dt)
            out["O"][b, h] = O
            out["dV"][b, h] = _r(_r(P, dt).T @ do, dt)
            out["dQ"][b, h] = _r(scale * (dS @ k), dt)
            out["dK"][b, h] = _r(scale * (dS.T @ q), dt)
    return out


# Offsets (natural-log units) of the softmax reference point above the row maximum.  Rounding to a
# binary floating-point format commutes with scaling by two, so the realisation depends on the
# offset modulo ln 2 only: eight equally spaced points cover that period.  (Three arbitrary points
# were too few: a row whose probabilities are dominated by a few keys gets an O that is off by the
# rounding error of those few P' as a whole, Delta = rowsum(dO (.) O) inherits it, and dQ of that
# row moves by (error of Delta) * scale * P K -- a figure that, on a random input, only some
# reference points show.)
REF_SHIFTS = tuple(float(k) / 8.0 * float(np.log(2.0)) for k in range(8))


def attn_realisations(c):
    """The ideal pipeline for each reference point of REF_SHIFTS: a list of attn() results."""
    return [attn(c, sh) for sh in REF_SHIFTS]
