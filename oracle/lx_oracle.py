"""ctypes front end of the CPU oracle (oracle/lx_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  Marshals numpy arrays; all arithmetic is in the
C++ file.  Takes dense block masks (one byte per block) like the definition.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        if os.environ.get("LX_ORACLE_SANITIZED") == "1":     # the ASan + UBSan build (CPU tests)
            path = _build.build_sanitized(force=False)
        else:
            path = _build.build(force=False)
        _lib = C.CDLL(path)
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint8))


def _f64_out(shape):
    a = np.empty(shape, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def mask_compact(mask, transpose=False):
    """Row-compressed active-block list of a 2-D byte mask.  With
    transpose=True the list is built over the columns (column-compressed)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    R, Cc = mask.shape
    if transpose:
        rows, cols, rs, cs = Cc, R, 1, Cc
    else:
        rows, cols, rs, cs = R, Cc, Cc, 1
    row_ptr = np.empty(rows + 1, dtype=np.int32)
    col_idx = np.empty(max(rows * cols, 1), dtype=np.int32)
    lib().lxo_mask_compact(
        mask.ctypes.data_as(C.POINTER(C.c_uint8)), C.c_int32(rows),
        C.c_int32(cols), C.c_int64(rs), C.c_int64(cs),
        row_ptr.ctypes.data_as(C.POINTER(C.c_int32)),
        col_idx.ctypes.data_as(C.POINTER(C.c_int32)))
    return row_ptr, col_idx[:row_ptr[-1]].copy()


def ffn_fwd(X, W_up, W_down, mask, tile_t, blk_n, b_up=None, b_down=None):
    """Returns (H [T,F], Y [T,d]) in float64."""
    T, d = X.shape
    F = W_up.shape[0]
    assert W_up.shape == (F, d) and W_down.shape == (d, F)
    assert mask.shape == (T // tile_t, F // blk_n)
    X, pX = _f32(X)
    W_up, pU = _f32(W_up)
    W_down, pD = _f32(W_down)
    mask, pM = _u8(mask)
    pbu = pbd = None
    if b_up is not None:
        b_up, pbu = _f32(b_up)
    if b_down is not None:
        b_down, pbd = _f32(b_down)
    H, pH = _f64_out((T, F))
    Y, pY = _f64_out((T, d))
    lib().lxo_ffn_fwd(C.c_int32(T), C.c_int32(d), C.c_int32(F),
                      C.c_int32(tile_t), C.c_int32(blk_n), pX, pU, pbu, pD,
                      pbd, pM, pH, pY)
    return H, Y


def ffn_bwd_dx(dY, W_up, W_down, mask, act, tile_t, blk_n):
    """act: [T,F] activation map (non-zero where the forward Z was > 0).
    Returns (dZ [T,F], dX [T,d]) in float64."""
    T, d = dY.shape
    F = W_up.shape[0]
    dY, pdY = _f32(dY)
    W_up, pU = _f32(W_up)
    W_down, pD = _f32(W_down)
    mask, pM = _u8(mask)
    act, pA = _u8(act)
    assert act.shape == (T, F)
    dZ, pdZ = _f64_out((T, F))
    dX, pdX = _f64_out((T, d))
    lib().lxo_ffn_bwd_dx(C.c_int32(T), C.c_int32(d), C.c_int32(F),
                         C.c_int32(tile_t), C.c_int32(blk_n), pdY, pU, pD, pM,
                         pA, pdZ, pdX)
    return dZ, dX


def _attn_args(Q, K, V, mask, head_active, blk):
    B, Hh, S, D = Q.shape
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.ndim == 3:
        mask = mask[None]
    mb = mask.shape[0]
    assert mask.shape == (mb, Hh, S // blk, S // blk) and mb in (1, B)
    return B, Hh, S, D, mask, mb


def attn_fwd(Q, K, V, mask, scale, causal, head_active=None, blk=64):
    """Returns (O [B,Hh,S,D], LSE [B,Hh,S]) in float64."""
    B, Hh, S, D, mask, mb = _attn_args(Q, K, V, mask, head_active, blk)
    Q, pQ = _f32(Q)
    K, pK = _f32(K)
    V, pV = _f32(V)
    pM = mask.ctypes.data_as(C.POINTER(C.c_uint8))
    pHa = None
    if head_active is not None:
        head_active, pHa = _u8(head_active)
    O, pO = _f64_out((B, Hh, S, D))
    L, pL = _f64_out((B, Hh, S))
    lib().lxo_attn_fwd(C.c_int32(B), C.c_int32(Hh), C.c_int32(S), C.c_int32(D),
                       C.c_double(scale), C.c_int32(int(causal)), pQ, pK, pV,
                       C.c_int32(blk), pM, C.c_int32(mb), pHa, pO, pL)
    return O, L


def attn_bwd(Q, K, V, dO, mask, scale, causal, head_active=None, blk=64):
    """Returns (dQ, dK, dV) [B,Hh,S,D] in float64."""
    B, Hh, S, D, mask, mb = _attn_args(Q, K, V, mask, head_active, blk)
    Q, pQ = _f32(Q)
    K, pK = _f32(K)
    V, pV = _f32(V)
    dO, pdO = _f32(dO)
    pM = mask.ctypes.data_as(C.POINTER(C.c_uint8))
    pHa = None
    if head_active is not None:
        head_active, pHa = _u8(head_active)
    dQ, pdQ = _f64_out((B, Hh, S, D))
    dK, pdK = _f64_out((B, Hh, S, D))
    dV, pdV = _f64_out((B, Hh, S, D))
    lib().lxo_attn_bwd(C.c_int32(B), C.c_int32(Hh), C.c_int32(S), C.c_int32(D),
                       C.c_double(scale), C.c_int32(int(causal)), pQ, pK, pV,
                       pdO, C.c_int32(blk), pM, C.c_int32(mb), pHa, pdQ, pdK,
                       pdV)
    return dQ, dK, dV


def mlp_predict(X, Wa, thr, group_rows=None):
    """MLP predictor of Sec. V-A: scores S = X Wa [T, nblk] (float64) and the
    block mask [T/group_rows, nblk] (uint8) = OR over the tokens of a group of
    (S > thr).  group_rows=None: one group holding all tokens."""
    T, d = X.shape
    nblk = Wa.shape[1]
    assert Wa.shape == (d, nblk)
    g = T if group_rows is None else group_rows
    assert T % g == 0
    X, pX = _f32(X)
    Wa, pW = _f32(Wa)
    S, pS = _f64_out((T, nblk))
    M = np.empty((T // g, nblk), dtype=np.uint8)
    lib().lxo_mlp_predict(C.c_int32(T), C.c_int32(d), C.c_int32(nblk), C.c_int32(g), pX, pW,
                          C.c_double(thr), pS, M.ctypes.data_as(C.POINTER(C.c_uint8)))
    return S, M


def combine_patterns(pool, head_pattern):
    """Dense multi-head block mask [Hm, nblk, nblk]: head h carries pool[head_pattern[h]]
    (no block for a negative entry).  pool: [P, nblk, nblk] bytes."""
    pool = np.ascontiguousarray(pool, dtype=np.uint8)
    P, nblk, n2 = pool.shape
    assert nblk == n2
    hp = np.ascontiguousarray(head_pattern, dtype=np.int32)
    out = np.empty((hp.shape[0], nblk, nblk), dtype=np.uint8)
    lib().lxo_attn_combine_patterns(
        C.c_int32(P), C.c_int32(nblk), pool.ctypes.data_as(C.POINTER(C.c_uint8)),
        C.c_int32(hp.shape[0]), hp.ctypes.data_as(C.POINTER(C.c_int32)),
        out.ctypes.data_as(C.POINTER(C.c_uint8)))
    return out


def ffn_lora_fwd(X, W_up, A, B, W_down, mask, tile_t, blk_n):
    """LoRA branch on the up-projection.  A [r,d], B [F,r].  Returns (U [T,r], H [T,F], Y [T,d])
    in float64."""
    T, d = X.shape
    F, r = B.shape
    assert W_up.shape == (F, d) and W_down.shape == (d, F) and A.shape == (r, d)
    assert mask.shape == (T // tile_t, F // blk_n)
    X, pX = _f32(X)
    W_up, pU = _f32(W_up)
    A, pA = _f32(A)
    B, pB = _f32(B)
    W_down, pD = _f32(W_down)
    mask, pM = _u8(mask)
    U, pu = _f64_out((T, r))
    H, pH = _f64_out((T, F))
    Y, pY = _f64_out((T, d))
    lib().lxo_ffn_lora_fwd(C.c_int32(T), C.c_int32(d), C.c_int32(F), C.c_int32(r), C.c_int32(tile_t),
                           C.c_int32(blk_n), pX, pU, pA, pB, pD, pM, pu, pH, pY)
    return U, H, Y


def ffn_lora_bwd(X, dY, W_up, A, B, W_down, mask, act, U, tile_t, blk_n):
    """Returns dict(dZ [T,F], G [T,r], dX [T,d], dA [r,d], dB [F,r]) in float64; U is the stored
    forward U (float64 array, possibly rounded by the caller), act the map [Z > 0]."""
    T, d = X.shape
    F, r = B.shape
    X, pX = _f32(X)
    dY, pdY = _f32(dY)
    W_up, pU = _f32(W_up)
    A, pA = _f32(A)
    B, pB = _f32(B)
    W_down, pD = _f32(W_down)
    mask, pM = _u8(mask)
    act, pact = _u8(act)
    U = np.ascontiguousarray(U, dtype=np.float64)
    assert act.shape == (T, F) and U.shape == (T, r)
    dZ, pdZ = _f64_out((T, F))
    G, pG = _f64_out((T, r))
    dX, pdX = _f64_out((T, d))
    dA, pdA = _f64_out((r, d))
    dB, pdB = _f64_out((F, r))
    lib().lxo_ffn_lora_bwd(C.c_int32(T), C.c_int32(d), C.c_int32(F), C.c_int32(r), C.c_int32(tile_t),
                           C.c_int32(blk_n), pX, pdY, pU, pA, pB, pD, pM, pact,
                           U.ctypes.data_as(C.POINTER(C.c_double)), pdZ, pG, pdX, pdA, pdB)
    return dict(dZ=dZ, G=G, dX=dX, dA=dA, dB=dB)
