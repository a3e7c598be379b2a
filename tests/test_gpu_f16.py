"""GPU parity of the IEEE-half element type (LX_F16: fp16 operands, fp32 accumulation -- the
parameter precision the paper trains with, Sec. VII-A) through every 16-bit entry point:
sparse FFN forward / input gradient, per-tile and shared lists, biases; block-sparse attention
forward / backward for both head sizes; the MLP predictor; the LoRA-branch FFN.  Same oracle,
same cases as the bfloat16 tests, inputs rounded to half instead; the gates are an eighth of
bfloat16's (three more significand bits)."""
import numpy as np
import pytest

import test_gpu_attn as A
import test_gpu_ffn as F
import test_gpu_lora as L
import test_gpu_predict as P
from paper_2510_15964_amd import inputs
from util import FRO, TOL, dev, host, rel_err_fro, rel_err_max, round_to

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lx():
    import torch
    assert torch.cuda.is_available()
    from paper_2510_15964_amd import lx
    return lx


@pytest.mark.parametrize("T,d,F_,density,seed", [
    (256, 256, 1024, 0.3, 111),     # several tiles, ragged per-row counts
    (192, 192, 704, 0.45, 112),     # d not a multiple of 256, 11 neuron blocks
    (128, 64, 320, 1.0, 113),       # dense
    (128, 128, 256, 0.0, 114),      # empty mask
])
def test_ffn_f16_matches_oracle(lx, oracle, T, d, F_, density, seed):
    c = inputs.ffn_bernoulli(T, d, F_, 64, 64, density, seed, dtype="f16", w_std=0.05)
    F.compare(lx, oracle, c)
    F.compare(lx, oracle, c, packed=False)


def test_ffn_f16_bias(lx, oracle):
    c = inputs.ffn_bernoulli(256, 128, 512, 64, 64, 0.4, 121, dtype="f16", w_std=0.1)
    rng = np.random.default_rng(3)
    c["b_up"] = round_to(rng.standard_normal(c["F"]) * 0.1, "f16")
    c["b_down"] = round_to(rng.standard_normal(c["d"]), "f16")
    c["mask"][1, :] = 0
    got, _ = F.compare(lx, oracle, c, bias=True)
    assert np.array_equal(got["Y"][64:128], np.broadcast_to(c["b_down"], (64, c["d"])))


def test_ffn_f16_bench_widths(lx, oracle):
    """OPT-1.3B widths, planted-support recipe of configs[1] with half-precision rounding, 256
    tokens (the oracle's fp64 loops set the size)."""
    c = inputs.ffn_planted_support(256, 2048, 8192, 64, 64, 0.5, 4.0, seed=2001, dtype="f16")
    F.compare(lx, oracle, c)


def test_ffn_f16_differs_from_bf16_only_by_rounding(lx, oracle):
    """The same fp16-representable problem run as bf16 would have to re-round the inputs; run as
    fp16 its error against the oracle is several times smaller than the bf16 run of the
    bf16-rounded problem -- the element type really is the one asked for."""
    c16 = inputs.ffn_bernoulli(256, 256, 1024, 64, 64, 0.3, 131, dtype="f16", w_std=0.05)
    cbf = inputs.ffn_bernoulli(256, 256, 1024, 64, 64, 0.3, 131, dtype="bf16", w_std=0.05)
    e16 = rel_err_fro(F.run_gpu(lx, c16)["Y"], F.run_oracle(oracle, c16)["Y"])
    ebf = rel_err_fro(F.run_gpu(lx, cbf)["Y"], F.run_oracle(oracle, cbf)["Y"])
    print(f"Frobenius error of Y: f16 {e16:.2e}, bf16 {ebf:.2e}", flush=True)
    assert e16 < ebf / 4


@pytest.mark.parametrize("kw,seed", [
    (dict(B=2, Hh=3, S=256, D=64, density=0.4), 201),
    (dict(B=1, Hh=2, S=320, D=128, density=0.5), 202),
    (dict(B=2, Hh=2, S=192, D=64, density=1.0), 203),
    (dict(B=1, Hh=4, S=256, D=64, density=0.3, causal=False), 204),
    (dict(B=2, Hh=4, S=128, D=128, density=0.5, head_keep=0.5), 205),
    (dict(B=1, Hh=2, S=128, D=64, density=0.0), 206),
])
def test_attn_f16_matches_oracle(lx, oracle, kw, seed):
    c = inputs.attn_blocks(seed=seed, dtype="f16", **kw)
    A.check(A.run_gpu(lx, c), A.run_oracle(oracle, c), f"f16 {kw}", dtype="f16")


def test_attn_f16_config3_shape_sampled_heads(lx, oracle):
    """configs[2]'s shape and mask recipe with half-precision tensors, full size on the GPU;
    the oracle checks sampled (batch, head) pairs."""
    c = inputs.attn_blocks(8, 32, 1024, 64, 0.30, seed=3001, dtype="f16", head_keep=7 / 8)
    got = A.run_gpu(lx, c)
    on = np.nonzero(c["head_active"])[0]
    for b, h in ((0, int(on[0])), (5, int(on[len(on) // 2])), (7, int(on[-1]))):
        sub = dict(c, B=1, Hh=1, head_active=np.ones(1, np.uint8),
                   mask=np.ascontiguousarray(c["mask"][:, h:h + 1]),
                   **{k: np.ascontiguousarray(c[k][b:b + 1, h:h + 1]) for k in ("Q", "K", "V", "dO")})
        ref = A.run_oracle(oracle, sub)
        g = {k: v[b:b + 1, h:h + 1] for k, v in got.items()}
        A.check(g, ref, f"f16 configs[2] shape b={b} h={h}", dtype="f16")
    off = np.nonzero(c["head_active"] == 0)[0]
    for k in ("O", "dQ", "dK", "dV"):
        assert not got[k][:, off].any()


@pytest.mark.parametrize("T,d,nblk,group,thr,seed", [
    (256, 128, 64, 64, 2.5, 301),
    (512, 256, 128, 512, 3.1, 302),
    (2048, 128, 2048, 256, 2.8, 306),
    (8192, 64, 384, 1024, 3.2, 307),
])
def test_predict_f16_matches_oracle(lx, oracle, T, d, nblk, group, thr, seed):
    X, Wa_t = P._case(T, d, nblk, seed, dtype="f16")
    got, M = P._check(lx, oracle, X, Wa_t, thr, group, dtype="f16")
    assert 0.02 < M.mean() < 0.98


@pytest.mark.parametrize("T,d,F_,r,density,seed,rows", [
    (256, 128, 512, 16, 0.4, 401, None),
    (512, 256, 1024, 64, 0.2, 402, None),
    (512, 128, 768, 16, 0.4, 405, 2),          # two list rows for eight tiles
    (512, 2048, 8192, 16, 0.11, 409, None),    # OPT-1.3B widths: the split-K / split-tile paths
])
def test_lora_f16_matches_oracle(lx, oracle, T, d, F_, r, density, seed, rows):
    c = L.make_case(T, d, F_, r, density, seed, rows=rows, dtype="f16")
    got, ref = L.run_both(lx, oracle, c)
    L.check(got, ref, f"f16 T={T} d={d} F={F_} r={r}", dtype="f16")
    assert not got["dA"][r:].any() and not got["dB"][:, r:].any() and not got["U"][:, r:].any()
