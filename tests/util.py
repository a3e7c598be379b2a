"""Shared helpers for the parity tests (no operator arithmetic)."""
from __future__ import annotations

import numpy as np

# Gates, identical for every output tensor:
#   TOL bounds rel_err_max = max|g - r| / max|r|   ("max relative error": the
#       largest error against the largest reference magnitude of the tensor),
#   FRO bounds rel_err_fro = ||g - r||_F / ||r||_F (about two bf16 unit
#       roundoffs of 2^-9: one for the factor that is rounded before the second
#       product -- H, dZ, P, dS -- and one for the rounded output).
# rel_err, the element-wise error with an rms floor, is printed next to them and
# also gated for fp32.  It cannot gate bf16 at 2e-2: outputs whose rows differ
# in scale by an order of magnitude (a query with one allowed key vs. hundreds;
# the gate channels of the planted-support FFN input) read 0.03-0.06 on it even
# for an ideal pipeline that is exact apart from rounding P / dS / dZ to bf16.
# IEEE half ("f16") carries three more significand bits than bfloat16: its gates are an
# eighth of bfloat16's.
TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 2.5e-3}
FRO = {"f32": 2e-6, "bf16": 5e-3, "f16": 6.25e-4}
# 16-bit runs: the element-wise error with an rms floor (rel_err) is gated against what the ideal
# 16-bit pipeline (tests/emulate16.py: one rounding of the intermediate factor, one of the output,
# everything else exact) loses on the same input: at most EMUL_FACTOR times that figure.  The figure
# is the maximum of ~10^5 rounding errors and so depends on which values get rounded; equally valid
# realisations of the ideal pipeline differ by up to a factor of two in it (test_emulated_gate.py),
# hence a factor of one half above the envelope of the emulated realisations rather than a quarter
# (largest ratio seen: 1.30 over 1920 tensors of random attention cases, 1.23 over the GPU tests).
EMUL_FACTOR = 1.5


def rel_err(got, ref) -> float:
    """max_i |g_i - r_i| / max(|r_i|, rms(r)).  Plain element-wise relative
    error is undefined at the many exact zeros of masked outputs, so small
    elements are measured against the tensor's rms."""
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(r * r)))
    if rms == 0.0:
        return float(np.max(np.abs(g)))       # reference is all zero: must match exactly
    return float(np.max(np.abs(g - r) / np.maximum(np.abs(r), rms)))


def rel_err_rows(got, ref) -> float:
    """max over the rows (vectors along the last axis) of max|g - r| / max|r| of that row: every
    row is measured against its OWN scale, so a row of small magnitude (a query with one allowed
    key, a gate channel) cannot hide behind the large ones.  Rows whose largest reference magnitude
    is below ROW_FLOOR times the tensor's are measured against that floor (their values are
    cancellation residue of sums whose terms are that much larger)."""
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return 0.0
    top = float(np.max(np.abs(r)))
    if top == 0.0:
        return float(np.max(np.abs(g)))
    num = np.max(np.abs(g - r), axis=-1)
    den = np.maximum(np.max(np.abs(r), axis=-1), ROW_FLOOR * top)
    return float(np.max(num / den))


ROW_FLOOR = 1e-3
# largest ratio of the kernels' per-row figure to the ideal pipeline's: 1.04 over the tensors of the
# GPU tests, 1.26 over random attention cases (most are exactly 1: the worst row is an
# output-rounding error either way)
ROW_FACTOR = EMUL_FACTOR


def assert_within_emulated(got, ref, emul, name, factor=EMUL_FACTOR):
    """rel_err(got, ref) <= factor * rel_err(emul, ref): the kernel's element-wise error against the
    oracle is at most `factor` times the ideal 16-bit pipeline's on the same input; likewise the
    per-row figure rel_err_rows at ROW_FACTOR.  emul: one emulated tensor, or a list of equally
    valid realisations of the pipeline, whose largest figure counts.  Returns the tensor-wide
    figures."""
    emuls = emul if isinstance(emul, (list, tuple)) else [emul]
    e_got, e_emul = rel_err(got, ref), max(rel_err(e, ref) for e in emuls)
    r_got, r_emul = rel_err_rows(got, ref), max(rel_err_rows(e, ref) for e in emuls)
    print(f"   [{name}] rms-floored {e_got:.5f} ideal pipeline {e_emul:.5f} ratio "
          f"{e_got / max(e_emul, 1e-30):.3f}; per row {r_got:.5f} ideal {r_emul:.5f} ratio "
          f"{r_got / max(r_emul, 1e-30):.3f}", flush=True)
    assert e_got <= factor * e_emul, (name, "rms-floored error", e_got, "ideal pipeline", e_emul)
    assert r_got <= ROW_FACTOR * r_emul, (name, "per-row error", r_got, "ideal pipeline", r_emul)
    return e_got, e_emul


def rel_err_max(got, ref) -> float:
    """max_i |g_i - r_i| / max_j |r_j|."""
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape
    den = float(np.max(np.abs(r))) if r.size else 0.0
    num = float(np.max(np.abs(g - r))) if r.size else 0.0
    return num if den == 0.0 else num / den


def rel_err_fro(got, ref) -> float:
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    den = float(np.linalg.norm(r))
    num = float(np.linalg.norm(g - r))
    return num if den == 0.0 else num / den


def torch_dtype(name):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[name]


def lx_dtype(lx, name):
    """The library's dtype code of a run dtype name."""
    return {"f32": lx.LX_F32, "bf16": lx.LX_BF16, "f16": lx.LX_F16}[name]


def dev(a, dtype="f32"):
    """numpy float32 (already representable in `dtype`) -> device tensor."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch_dtype(dtype)).contiguous()


def host(t):
    return t.detach().float().cpu().numpy()


def round_to(a, dtype):
    """Round an fp64/fp32 array to the run dtype, returned as float32."""
    from paper_2510_15964_amd.inputs import bf16_round, f16_round
    a32 = np.asarray(a, dtype=np.float32)
    return bf16_round(a32) if dtype == "bf16" else f16_round(a32) if dtype == "f16" else a32


def compact_blocks(dense, mask, tile_t, blk_n):
    """Dense [T,F] -> compact [nnz, tile_t, blk_n] in row-major list order."""
    Tt, Fb = mask.shape
    v = dense.reshape(Tt, tile_t, Fb, blk_n).transpose(0, 2, 1, 3)
    return np.ascontiguousarray(v[mask.astype(bool)])


def expand_blocks(compact, mask, tile_t, blk_n, fill=0.0):
    Tt, Fb = mask.shape
    out = np.full((Tt, Fb, tile_t, blk_n), fill, dtype=compact.dtype)
    out[mask.astype(bool)] = compact
    return np.ascontiguousarray(out.transpose(0, 2, 1, 3)).reshape(Tt * tile_t, Fb * blk_n)
