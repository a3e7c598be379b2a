"""GPU parity on seeded random shapes, densities and options (a sweep over combinations the
hand-picked cases of the other files do not enumerate)."""
import numpy as np
import pytest

from paper_2510_15964_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lx():
    import torch
    assert torch.cuda.is_available()
    from paper_2510_15964_amd import lx
    return lx


@pytest.mark.parametrize("seed", [101, 202, 303])
def test_ffn_random_shapes(lx, oracle, seed):
    from test_gpu_ffn import compare
    rng = np.random.default_rng(seed)
    for _ in range(6):
        T, d, F = (64 * int(rng.integers(1, 9)), 64 * int(rng.integers(1, 6)), 64 * int(rng.integers(1, 12)))
        rho = float(rng.choice([0.0, 0.05, 0.3, 0.7, 1.0]))
        c = inputs.ffn_bernoulli(T, d, F, 64, 64, rho, int(rng.integers(1, 10 ** 6)),
                                 dtype=str(rng.choice(["bf16", "f16"])), w_std=0.05)
        compare(lx, oracle, c)


@pytest.mark.parametrize("seed", [111, 222, 333])
def test_attention_random_shapes(lx, oracle, seed):
    from test_gpu_attn import check, run_gpu, run_oracle
    rng = np.random.default_rng(seed)
    try:
        for _ in range(6):
            B, Hh, S = int(rng.integers(1, 3)), int(rng.integers(1, 5)), 64 * int(rng.integers(1, 10))
            D = int(rng.choice([64, 128]))
            dtype = str(rng.choice(["bf16", "f16"]))
            a = inputs.attn_blocks(B, Hh, S, D, float(rng.choice([0.0, 0.1, 0.4, 1.0])),
                                   int(rng.integers(1, 10 ** 6)), dtype=dtype,
                                   causal=bool(rng.integers(0, 2)), head_keep=float(rng.choice([1.0, 0.6])),
                                   force_diagonal=bool(rng.integers(0, 2)), mask_batch=int(rng.choice([1, B])))
            lx.lx_attn_set_rows_per_workgroup(int(rng.choice([0, 1, 3, 8])))
            check(run_gpu(lx, a), run_oracle(oracle, a), f"random {dtype} B={B} H={Hh} S={S} D={D}",
                  dtype=dtype)
    finally:
        lx.lx_attn_set_rows_per_workgroup(0)


@pytest.mark.parametrize("seed", [131, 242])
def test_attention_random_shapes_fp32(lx, oracle, seed):
    """The fp32 correctness kernels on random shapes and options, at the fp32 gates."""
    from test_gpu_attn import check, run_gpu, run_oracle
    rng = np.random.default_rng(seed)
    try:
        for _ in range(5):
            B, Hh, S = int(rng.integers(1, 3)), int(rng.integers(1, 5)), 64 * int(rng.integers(1, 8))
            D = int(rng.choice([64, 128]))
            a = inputs.attn_blocks(B, Hh, S, D, float(rng.choice([0.0, 0.1, 0.4, 1.0])),
                                   int(rng.integers(1, 10 ** 6)), dtype="f32",
                                   causal=bool(rng.integers(0, 2)), head_keep=float(rng.choice([1.0, 0.6])),
                                   force_diagonal=bool(rng.integers(0, 2)), mask_batch=int(rng.choice([1, B])))
            layout = str(rng.choice(["bhsd", "bshd"]))
            check(run_gpu(lx, a, layout=layout), run_oracle(oracle, a),
                  f"random f32 B={B} H={Hh} S={S} D={D} {layout}", dtype="f32")
    finally:
        lx.lx_attn_set_rows_per_workgroup(0)


@pytest.mark.parametrize("seed", [121, 232])
def test_lora_random_shapes(lx, oracle, seed):
    from test_gpu_lora import check, make_case, run_both
    rng = np.random.default_rng(seed)
    for _ in range(5):
        Tt = int(rng.integers(1, 9))
        d, F = 64 * int(rng.integers(1, 6)), 64 * int(rng.integers(1, 12))
        r = int(rng.choice([1, 4, 16, 33, 64]))
        rows = int(rng.choice([g for g in range(1, Tt + 1) if Tt % g == 0]))   # list rows: a divisor of the tiles
        dtype = str(rng.choice(["bf16", "f16"]))
        c = make_case(64 * Tt, d, F, r, float(rng.choice([0.0, 0.1, 0.4, 1.0])), int(rng.integers(1, 10 ** 6)),
                      rows=None if rows == Tt else rows, dtype=dtype)
        got, ref = run_both(lx, oracle, c)
        check(got, ref, f"random {dtype} T={64 * Tt} d={d} F={F} r={r} rows={rows}", dtype=dtype)
