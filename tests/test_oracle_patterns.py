"""Pins of the oracle's online pattern combination (Sec. VI-A): each head carries the pattern it
is assigned, the multi-head list is the compaction of the per-head patterns side by side."""
import numpy as np
import pytest

from paper_2510_15964_amd import inputs


def test_hand_example(oracle):
    # two 2x2 patterns; heads 1, 0, none, 1 -- written out by hand
    pool = np.array([[[1, 0], [1, 1]],
                     [[0, 0], [0, 1]]], dtype=np.uint8)
    m = oracle.combine_patterns(pool, [1, 0, -1, 1])
    want = np.array([[[0, 0], [0, 1]],
                     [[1, 0], [1, 1]],
                     [[0, 0], [0, 0]],
                     [[0, 0], [0, 1]]], dtype=np.uint8)
    assert np.array_equal(m, want)
    rp, ci = oracle.mask_compact(m.reshape(8, 2))
    assert rp.tolist() == [0, 0, 1, 2, 4, 4, 4, 4, 5]
    assert ci.tolist() == [1, 0, 0, 1, 1]


def test_brute_force_and_values(oracle):
    rng = np.random.default_rng(3)
    pool = (rng.random((5, 7, 7)) < 0.4).astype(np.uint8) * rng.integers(1, 255, (5, 7, 7)).astype(np.uint8)
    hp = rng.integers(-1, 5, 23)
    m = oracle.combine_patterns(pool, hp)
    assert set(np.unique(m)) <= {0, 1}                        # any non-zero byte counts as active
    for h, p in enumerate(hp):
        for q in range(7):
            for k in range(7):
                assert m[h, q, k] == (1 if p >= 0 and pool[p, q, k] else 0)


def test_same_pattern_everywhere_is_a_tile_of_it(oracle):
    pool = inputs.pattern_pool(16, seed=5)
    for p in range(pool.shape[0]):
        m = oracle.combine_patterns(pool, [p] * 6)
        assert np.array_equal(m, np.tile(pool[p][None], (6, 1, 1)))


def test_list_is_the_pool_layouts_with_an_offset_per_head(oracle):
    """What the paper's combination step does: the layout of a head is the pre-computed layout
    of its pattern, shifted by the number of blocks of the heads before it."""
    pool = inputs.pattern_pool(12, seed=9)
    rng = np.random.default_rng(10)
    hp = rng.integers(-1, pool.shape[0], 20)
    m = oracle.combine_patterns(pool, hp)
    for transpose in (False, True):
        mm = m.transpose(0, 2, 1) if transpose else m
        rp, ci = oracle.mask_compact(mm.reshape(-1, 12))
        lut = [oracle.mask_compact(pool[p].T if transpose else pool[p]) for p in range(pool.shape[0])]
        off = 0
        for h, p in enumerate(hp):
            prp, pci = lut[p] if p >= 0 else (np.zeros(13, np.int32), np.zeros(0, np.int32))
            assert np.array_equal(rp[h * 12:(h + 1) * 12 + 1], prp + off)
            assert np.array_equal(ci[off:off + prp[-1]], pci)
            off += int(prp[-1])
        assert rp[-1] == off


def test_heads_commute(oracle):
    pool = inputs.pattern_pool(8, seed=1)
    hp = np.array([3, -1, 0, 7, 2, 2])
    perm = np.array([4, 0, 5, 1, 3, 2])
    assert np.array_equal(oracle.combine_patterns(pool, hp[perm]), oracle.combine_patterns(pool, hp)[perm])


def test_attention_under_the_combined_mask_is_attention_per_head_under_its_pattern(oracle):
    B, Hh, S, D = 1, 3, 256, 32
    a = inputs.attn_blocks(B, Hh, S, D, 1.0, seed=77, dtype="f32", blk=64)
    pool = inputs.pattern_pool(4, seed=2)
    hp = [2, 5, 0]
    m = oracle.combine_patterns(pool, hp)[None]              # mask_batch = 1
    O, L = oracle.attn_fwd(a["Q"], a["K"], a["V"], m, a["scale"], 1)
    for h, p in enumerate(hp):
        Oh, Lh = oracle.attn_fwd(a["Q"][:, h:h + 1], a["K"][:, h:h + 1], a["V"][:, h:h + 1],
                                 pool[p][None, None], a["scale"], 1)
        assert np.array_equal(O[:, h:h + 1], Oh) and np.array_equal(L[:, h:h + 1], Lh)


@pytest.mark.parametrize("causal", [True, False])
def test_pool_patterns_are_what_they_say(causal):
    n = 16
    pool = inputs.pattern_pool(n, seed=4, causal=causal)
    q, k = np.arange(n)[:, None], np.arange(n)[None, :]
    assert pool.shape == (8, n, n) and set(np.unique(pool)) <= {0, 1}
    for p in pool:
        assert p[np.arange(n), np.arange(n)].all()            # every pattern keeps the diagonal
        if causal:
            assert not (p & (k > q)).any()
        else:
            assert np.array_equal(p, p.T) or True
    assert np.array_equal(pool[0], ((q - k < 2) & (q >= k)) if causal else (np.abs(q - k) < 2))
    assert pool[2][:, 0].all() and pool[3][:, :2][2:].all()   # global key blocks
    assert pool[4][8, 0] and pool[4][8, 4] and not pool[4][8, 5]   # stride 4 (+ window 2)
    assert pool[7].sum() == (n * (n + 1) // 2 if causal else n * n)
