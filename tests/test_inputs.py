"""Host-side checks of the seeded input generators (no GPU): the storage roundings agree with
torch's conversions bit for bit, the generators are deterministic, and the structures they
promise (causal block masks, planted ReLU support, pattern pools, zero-padded LoRA matrices)
hold."""
import numpy as np
import torch

from paper_2510_15964_amd import inputs


def _samples():
    rng = np.random.default_rng(7)
    x = np.concatenate([
        rng.standard_normal(4096).astype(np.float32),
        (rng.standard_normal(4096) * 1e-6).astype(np.float32),        # half: subnormal range
        np.clip(rng.standard_normal(1024) * 3e4, -6.5e4, 6.5e4).astype(np.float32),   # half: top of the range
        np.array([0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -9, 1.0 + 3 * 2.0 ** -9,   # bf16 ties
                  1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -24, 2.0 ** -25, 65504.0], np.float32)])
    return x


def test_bf16_round_matches_torch():
    x = _samples()
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(inputs.bf16_round(x).view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(inputs.bf16_bits(x), (ref.view(np.uint32) >> 16).astype(np.uint16))


def test_f16_round_matches_torch():
    x = _samples()
    ref = torch.from_numpy(x).to(torch.float16).to(torch.float32).numpy()
    assert np.array_equal(inputs.f16_round(x).view(np.uint32), ref.view(np.uint32))


def test_generators_are_deterministic_and_representable():
    for dtype, rnd in (("bf16", inputs.bf16_round), ("f16", inputs.f16_round)):
        a = inputs.ffn_bernoulli(128, 64, 256, 64, 64, 0.3, 5, dtype=dtype)
        b = inputs.ffn_bernoulli(128, 64, 256, 64, 64, 0.3, 5, dtype=dtype)
        for k in ("X", "W_up", "W_down", "dY", "mask"):
            assert np.array_equal(a[k], b[k])
        for k in ("X", "W_up", "W_down", "dY"):
            assert np.array_equal(rnd(a[k]), a[k])                     # already representable
        q = inputs.attn_blocks(1, 2, 192, 64, 0.4, 6, dtype=dtype)
        for k in ("Q", "K", "V", "dO"):
            assert np.array_equal(rnd(q[k]), q[k])
    c = inputs.ffn_bernoulli(128, 64, 256, 64, 64, 0.3, 6, dtype="bf16")
    assert not np.array_equal(a["X"], c["X"])                          # another seed, other values


def test_causal_block_masks_never_list_a_block_above_the_diagonal():
    a = inputs.attn_blocks(2, 4, 512, 64, 0.5, 9, causal=True, force_diagonal=True)
    m = a["mask"]                                                      # [mask_batch, Hh, nb, nb]
    for h in range(m.shape[1]):
        assert not np.triu(m[0, h], 1).any()
        assert m[0, h].diagonal().all()                                # forced diagonal
    p = inputs.pattern_pool(16, seed=3, causal=True)
    for pat in p:
        assert not np.triu(pat, 1).any()


def test_planted_support_mask_is_the_block_level_relu_support():
    for dtype in ("bf16", "f16"):
        c = inputs.ffn_planted_support(256, 256, 512, 64, 64, 0.5, 4.0, seed=11, dtype=dtype)
        Z = c["X"].astype(np.float64) @ c["W_up"].astype(np.float64).T
        act = (Z > 0).reshape(4, 64, 8, 64).any(axis=(1, 3))
        assert np.array_equal(act, c["mask"].astype(bool))


def test_lora_matrices_are_zero_padded_to_rank_64():
    lo = inputs.lora_matrices(128, 256, 16, seed=2)
    assert lo["A_pad"].shape == (64, 128) and lo["B_pad"].shape == (256, 64)
    assert not lo["A_pad"][16:].any() and not lo["B_pad"][:, 16:].any()
    assert lo["A_pad"][:16].any() and lo["B_pad"][:, :16].any()
