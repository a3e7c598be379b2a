"""Seeded synthetic workloads for the Dynamic-aware Operator.

This module only draws random numbers and arranges them into tensors and
block masks.  It contains none of the operator's arithmetic and imports
neither the CPU oracle nor the HIP binding; both sides of every parity test
are fed from here.

The shapes are OPT layer shapes (Table "Models for evaluation") and the mask
structure follows the qualitative description of Sec. IV: block-wise MLP
sparsity with strongly skewed per-neuron activity, and head-specific block
masks for attention.  They stand in for OPT weights and the E2E / Alpaca
activations used in Sec. VII, which are not available here.

All arrays are numpy float32.  For dtype "bf16" (or "f16") every value is rounded
to the nearest bfloat16 (IEEE half; ties to even) and then widened again, so that a
16-bit device tensor and the float32 array given to the oracle hold identical numbers.
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# bfloat16 helpers (storage format only)
# ----------------------------------------------------------------------------


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bfloat16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16, returned widened to float32."""
    b = bf16_bits(x).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).reshape(np.shape(x))


def f16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest IEEE half (ties to even), returned widened to float32."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_round(x)
    if dtype == "f16":
        return f16_round(x)
    if dtype == "f32":
        return x
    raise ValueError(f"dtype must be 'f32', 'bf16' or 'f16', got {dtype!r}")


def _rng(seed: int, stream: int) -> np.random.Generator:
    # independent streams: X, W_up, W_down, dY, mask, Q, K, V, dO, heads ...
    return np.random.default_rng(np.random.SeedSequence([int(seed), int(stream)]))


def _normal(rng, shape, std, dtype):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return _store(a, dtype)


# ----------------------------------------------------------------------------
# FFN workloads
# ----------------------------------------------------------------------------


def ffn_bernoulli(T, d, F, tile_t, blk_n, density, seed, dtype="f32",
                  w_std=0.02):
    """Generic data, iid Bernoulli(density) block mask [T/tile_t, F/blk_n]."""
    assert T % tile_t == 0 and F % blk_n == 0
    Tt, Fb = T // tile_t, F // blk_n
    X = _normal(_rng(seed, 0), (T, d), 1.0, dtype)
    W_up = _normal(_rng(seed, 1), (F, d), w_std, dtype)
    W_down = _normal(_rng(seed, 2), (d, F), w_std, dtype)
    dY = _normal(_rng(seed, 3), (T, d), 1.0, dtype)
    if density >= 1.0:
        mask = np.ones((Tt, Fb), dtype=np.uint8)
    elif density <= 0.0:
        mask = np.zeros((Tt, Fb), dtype=np.uint8)
    else:
        mask = (_rng(seed, 4).random((Tt, Fb)) < density).astype(np.uint8)
    return dict(kind="ffn", dtype=dtype, T=T, d=d, F=F, tile_t=tile_t,
                blk_n=blk_n, X=X, W_up=W_up, W_down=W_down, dY=dY, mask=mask)


def ffn_planted_support(T, d, F, tile_t, blk_n, beta_a, beta_b, seed,
                        dtype="bf16", w_std=0.02):
    """Block mask that IS the block-level support of ReLU(X W_up^T).

    Per-neuron firing probabilities p_f ~ Beta(beta_a, beta_b) are sorted so
    that hot and cold neurons cluster into blocks; block j fires in a token
    tile with probability mean(p_f over the block).  The last Tt = T/tile_t
    input channels are gates: channel i carries gamma on the tokens of tile i
    and zero elsewhere, and a neuron of a block that is inactive in tile i has
    weight -beta on that channel.  With gamma*beta twelve standard deviations
    of the generic pre-activation, every pre-activation of an inactive block
    is negative, so the true ReLU support is exactly the drawn mask at block
    granularity (tests verify this on the oracle's dense forward pass).
    """
    assert T % tile_t == 0 and F % blk_n == 0
    Tt, Fb = T // tile_t, F // blk_n
    G = Tt
    assert d > G + 8, "need generic channels besides the gates"
    rm = _rng(seed, 4)
    p_f = np.sort(rm.beta(beta_a, beta_b, size=F))[::-1]
    p_blk = p_f.reshape(Fb, blk_n).mean(axis=1)
    # spread hot blocks over the neuron axis (deterministic shuffle) so that
    # the active list is not simply a prefix
    perm = _rng(seed, 5).permutation(Fb)
    p_blk = p_blk[perm]
    mask = (rm.random((Tt, Fb)) < p_blk[None, :]).astype(np.uint8)

    X = _normal(_rng(seed, 0), (T, d), 1.0, dtype)
    W_up = _normal(_rng(seed, 1), (F, d), w_std, dtype)
    W_down = _normal(_rng(seed, 2), (d, F), w_std, dtype)
    dY = _normal(_rng(seed, 3), (T, d), 1.0, dtype)

    sigma_c = w_std * np.sqrt(float(d - G))
    gamma = np.float32(4.0)
    beta = _store(np.array([12.0 * sigma_c / gamma], np.float32), dtype)[0]
    X[:, d - G:] = 0.0
    tile_of_token = np.arange(T) // tile_t
    X[np.arange(T), d - G + tile_of_token] = gamma
    # W_up[f, d-G+i] = 0 if mask[i, f//blk_n] else -beta
    gate = np.where(mask.T.astype(bool), np.float32(0.0), -np.float32(beta))  # [Fb, Tt]
    W_up[:, d - G:] = np.repeat(gate, blk_n, axis=0)
    return dict(kind="ffn", dtype=dtype, T=T, d=d, F=F, tile_t=tile_t,
                blk_n=blk_n, X=X, W_up=W_up, W_down=W_down, dY=dY, mask=mask,
                planted=True)


# ----------------------------------------------------------------------------
# attention workloads
# ----------------------------------------------------------------------------


def attn_blocks(B, Hh, S, D, density, seed, dtype="bf16", causal=True,
                head_keep=1.0, force_diagonal=False, blk=64, mask_batch=1):
    """Q, K, V, dO ~ N(0,1); per-head Bernoulli block mask inside the causal
    region (blocks above the diagonal are never set when causal).

    force_diagonal keeps every diagonal block on and lowers the off-diagonal
    probability so that the expected density inside the causal region stays
    `density`.
    """
    assert S % blk == 0
    nb = S // blk
    shp = (B, Hh, S, D)
    Q = _normal(_rng(seed, 10), shp, 1.0, dtype)
    K = _normal(_rng(seed, 11), shp, 1.0, dtype)
    V = _normal(_rng(seed, 12), shp, 1.0, dtype)
    dO = _normal(_rng(seed, 13), shp, 1.0, dtype)
    rm = _rng(seed, 14)
    u = rm.random((mask_batch, Hh, nb, nb))
    qi = np.arange(nb)[:, None]
    ki = np.arange(nb)[None, :]
    allowed = (ki <= qi) if causal else np.ones((nb, nb), dtype=bool)
    if force_diagonal and causal and density < 1.0:
        n_all = nb * (nb + 1) // 2
        n_off = n_all - nb
        p_off = max(0.0, (density * n_all - nb) / max(n_off, 1))
        m = (u < p_off) | (ki == qi)
    else:
        m = (u < density) if density < 1.0 else np.ones_like(u, dtype=bool)
    mask = (m & allowed).astype(np.uint8)
    if head_keep >= 1.0:
        head_active = np.ones(Hh, dtype=np.uint8)
    else:
        head_active = (_rng(seed, 15).random(Hh) < head_keep).astype(np.uint8)
        if head_active.sum() == 0:
            head_active[0] = 1
    return dict(kind="attn", dtype=dtype, B=B, Hh=Hh, S=S, D=D, blk=blk,
                causal=int(bool(causal)), scale=float(1.0 / np.sqrt(D)),
                Q=Q, K=K, V=V, dO=dO, mask=mask, mask_batch=mask_batch,
                head_active=head_active)


# ----------------------------------------------------------------------------
# the five named configurations
# ----------------------------------------------------------------------------

DENSITY_SWEEP = (0.05, 0.10, 0.20, 0.30, 0.50, 1.0)


def config1_ffn(seed=1000):
    """OPT-125m-shaped FFN, fp32, 32x32 blocks, Bernoulli 30 %."""
    return ffn_bernoulli(512, 768, 3072, 32, 32, 0.30, seed, dtype="f32")


def config2_ffn(seed=2000):
    """OPT-1.3B-shaped FFN, bf16, 64x64 blocks, planted ReLU support with
    Beta(0.5, 4) neuron probabilities (about 11 % mean block density)."""
    return ffn_planted_support(4096, 2048, 8192, 64, 64, 0.5, 4.0, seed)


def config3_attn(seed=3000, force_diagonal=False, dtype="bf16"):
    """OPT-1.3B-shaped causal attention, bf16, 30 % of causal 64x64 blocks,
    heads kept with probability 7/8."""
    return attn_blocks(8, 32, 1024, 64, 0.30, seed, dtype=dtype, head_keep=0.875,
                       force_diagonal=force_diagonal)


def config4_ffn(seed=4000):
    """OPT-6.7B-shaped FFN, planted support, Beta(0.5, 6)."""
    return ffn_planted_support(8192, 4096, 16384, 64, 64, 0.5, 6.0, seed)


def config4_attn(seed=4000):
    """OPT-6.7B-shaped attention, 25 % of causal blocks, all heads on."""
    return attn_blocks(4, 32, 2048, 128, 0.25, seed)


# ----------------------------------------------------------------------------
# attention patterns: the pool of Sec. VI-A is fed with dense block masks; these
# are the usual building blocks of the sparse-attention literature the paper
# cites (sliding window, global tokens, strided, random), as data
# ----------------------------------------------------------------------------

def pattern_local(nblk, w, causal=True):
    """Blocks within w block-diagonals of the diagonal (behind it only when causal)."""
    q, k = np.arange(nblk)[:, None], np.arange(nblk)[None, :]
    m = (q - k < w) & (q - k >= 0) if causal else (np.abs(q - k) < w)
    return m.astype(np.uint8)


def pattern_global(nblk, g, causal=True):
    """The first g key blocks are seen by every query block and the first g query blocks see
    every key block (up to the diagonal when causal)."""
    q, k = np.arange(nblk)[:, None], np.arange(nblk)[None, :]
    m = (k < g) | (q < g)
    if causal:
        m &= k <= q
    return m.astype(np.uint8)


def pattern_strided(nblk, s, causal=True):
    """Every s-th block diagonal."""
    q, k = np.arange(nblk)[:, None], np.arange(nblk)[None, :]
    m = (q - k) % s == 0
    if causal:
        m &= k <= q
    return m.astype(np.uint8)


def pattern_random(nblk, density, seed, causal=True):
    q, k = np.arange(nblk)[:, None], np.arange(nblk)[None, :]
    m = _rng(seed, 40).random((nblk, nblk)) < density
    if causal:
        m &= k <= q
    return m.astype(np.uint8)


def pattern_pool(nblk, seed=0, causal=True):
    """Eight patterns built from the atoms above: window, window + global (two widths each),
    window + strided, window + global + random, global + random, dense (causal)."""
    L, G, St, R = pattern_local, pattern_global, pattern_strided, pattern_random
    c = causal
    pool = [
        L(nblk, 2, c),
        L(nblk, 4, c),
        L(nblk, 2, c) | G(nblk, 1, c),
        L(nblk, 3, c) | G(nblk, 2, c),
        L(nblk, 2, c) | St(nblk, 4, c),
        L(nblk, 2, c) | G(nblk, 1, c) | R(nblk, 0.10, seed, c),
        L(nblk, 1, c) | G(nblk, 1, c) | R(nblk, 0.25, seed + 1, c),
        L(nblk, nblk, c),
    ]
    return np.stack(pool).astype(np.uint8)


def attn_patterns(B, Hh, S, D, seed, dtype="bf16", causal=True, probs=None, head_keep=1.0,
                  mask_batch=1):
    """Attention inputs whose block masks come from a pool: tensors as in attn_blocks, the pool
    of pattern_pool, and a seeded pattern id per (mask batch, head); heads dropped by head_keep
    get id -1 (no block).  The dense mask itself is not formed here."""
    c = attn_blocks(B, Hh, S, D, 1.0, seed, dtype=dtype, causal=causal, mask_batch=mask_batch)
    del c["mask"]
    pool = pattern_pool(S // 64, seed, causal)
    hp = _rng(seed, 41).choice(pool.shape[0], size=mask_batch * Hh, p=probs).astype(np.int32)
    if head_keep < 1.0:
        hp[_rng(seed, 42).random(mask_batch * Hh) >= head_keep] = -1
    c.update(pool=pool, head_pattern=hp)
    return c


def config3_patterns(seed=3100):
    """configs[2]'s shape with per-head patterns drawn so that the mean density inside the
    causal region is about 30 %, as in configs[2]."""
    return attn_patterns(8, 32, 1024, 64, seed, probs=(0.5, 0.08, 0.27, 0.03, 0.05, 0.05, 0.02, 0.0))


def lora_matrices(d, F, r, seed, b_std=0.02):
    """LoRA matrices A [r,d] ~ N(0, 1/d), B [F,r] ~ N(0, b_std^2) (a branch in mid-training: B is
    zero only at initialisation), bf16-representable, zero-padded to rank 64: A_pad [64,d],
    B_pad [F,64]."""
    A = np.zeros((64, d), np.float32)
    B = np.zeros((F, 64), np.float32)
    A[:r] = bf16_round((_rng(seed, 50).standard_normal((r, d)) / np.sqrt(d)).astype(np.float32))
    B[:, :r] = bf16_round((_rng(seed, 51).standard_normal((F, r)) * b_std).astype(np.float32))
    return dict(A_pad=A, B_pad=B, r=r)


def predictor_planted(d, nblk, density, seed, hot_scale=4.0, thr=6.5):
    """Predictor matrix Wa_t [nblk, d] (bf16-representable) whose block scores X Wa_t^T, for
    X ~ N(0,1), are N(0,1) for cold blocks and N(0, hot_scale^2) for a planted set of
    round(density * nblk) hot blocks.  Over thousands of tokens the largest score of a cold
    block stays below `thr` and that of a hot block far above it, so the mask reduced over the
    tokens is the planted set, with a wide margin around the threshold."""
    rng = _rng(seed, 20)
    hot = np.zeros(nblk, dtype=bool)
    hot[rng.permutation(nblk)[:int(round(density * nblk))]] = True
    W = rng.standard_normal((nblk, d)).astype(np.float32) / np.float32(np.sqrt(d))
    W[hot] *= np.float32(hot_scale)
    return dict(Wa_t=bf16_round(W), thr=float(thr), hot=hot)


def config5_ffn(density, seed=5000):
    """OPT-13B-shaped FFN, iid Bernoulli(density) blocks."""
    return ffn_bernoulli(4096, 5120, 20480, 64, 64, density,
                         seed + int(round(density * 100)), dtype="bf16")


def config5_attn(density, seed=5000):
    """OPT-13B-shaped attention, iid Bernoulli(density) causal blocks."""
    return attn_blocks(2, 40, 2048, 128, density,
                       seed + int(round(density * 100)))
