#!/usr/bin/env python3
"""Benchmark of the Dynamic-aware Operator hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input:
mask compaction, sparse FFN forward + input gradient, block-sparse attention
forward + backward.  Inputs (activations, frozen weights, dense byte masks) are
resident in HBM before the timed region; the frozen weights are repacked once,
outside it.

Workloads (recipes in paper_2510_15964_amd/inputs.py):
  opt1.3b_layer   default.  An OPT-1.3B-shaped layer over 8 x 1024 tokens:
                  attention = configs[2] (30 % of causal blocks), FFN =
                  configs[1]'s shape and recipe (planted ReLU support, ~10 %
                  blocks, a list per 64-token tile) applied to the 8192 tokens
                  in one call: 8 kernel launches per step.
  opt1.3b_layer_twocalls  the same layer with the FFN as two X[4096,2048] calls
                  (configs[1]'s own token count) that share the weights: 12 launches.
  The variants below keep the two-call FFN, the shape their parity tests cover:
  opt1.3b_layer_shared    the FFN masks predicted on the
                  device every step (MLP predictor, one list for all tokens of
                  a call: the paper's operating point, Sec. V-A).
  opt1.3b_layer_lora      a LoRA branch (rank 16) on the FFN
                  up-projection, including the gradients of A and B (Sec. II-C/D).
  opt1.3b_layer_f16       IEEE half precision (fp16 operands,
                  fp32 accumulation; the paper's parameter precision, Sec. VII-A).
  opt1.3b_layer_patterns  per-head attention patterns from
                  a pool, combined into the block lists on the device every
                  step (Sec. VI-A).
  opt1.3b_layer_hostw     the shared-list layer with the FFN weights in pinned host memory:
                  every call moves the listed neuron blocks to the device first (Sec. VII-B);
                  opt1.3b_layer_hostw_overlap = the same with the transfers on a second stream
                  under the attention kernels.
  config4         OPT-6.7B-shaped layer (configs[3]).
  config5:<rho>   OPT-13B-shaped layer at block density rho (configs[4]);
                  config5:<rho>:shared = the same with one FFN list for all token tiles
                  and four token tiles per FFN workgroup (the dense path at rho = 1).

Prints ONE JSON line.  `--sweep FILE` additionally runs the configs[4] density
sweep and writes one JSON line per density to FILE.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

METRIC = "sparse FFN+attn fwd+bwd-dX tokens/s and active-FLOP MFMA util @10/30% density"
PEAK_MFMA_BF16 = 2.5e15     # FLOP/s, dense MFMA on 16-bit operands (bf16 and fp16 alike), MI355X
PEAK_HBM = 8.0e12           # B/s
DEFAULT_WORKLOAD = "opt1.3b_layer"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ----------------------------------------------------------------------------
# workload construction (host) and device residency
# ----------------------------------------------------------------------------

def make_workload(name: str):
    from paper_2510_15964_amd import inputs
    if name == "opt1.3b_layer":
        # attention = configs[2]; FFN = configs[1]'s shape and planted-support recipe over the
        # layer's 8 x 1024 = 8192 tokens in ONE call (128 token tiles, a list per tile)
        f = inputs.ffn_planted_support(8192, 2048, 8192, 64, 64, 0.5, 4.0, seed=2000)
        a = inputs.config3_attn()
        ffn_calls = 1
    elif name == "opt1.3b_layer_twocalls":
        # the same layer with the FFN as two calls of configs[1]'s own 4096 tokens that share the
        # frozen weights: four more launches per step, and half as many token tiles share an XCD's L2
        f = inputs.ffn_planted_support(8192, 2048, 8192, 64, 64, 0.5, 4.0, seed=2000)
        a = inputs.config3_attn()
        ffn_calls = 2
    elif name == "opt1.3b_layer_shared":
        # the paper's own operating point (Sec. V-A): per FFN call ONE list of active neuron
        # blocks, predicted on the device from the call's tokens (scores, threshold, OR over
        # all tokens) and shared by all its token tiles; same shapes and density otherwise
        f = inputs.ffn_bernoulli(8192, 2048, 8192, 64, 64, 0.11, seed=2100, dtype="bf16")
        f["predictor"] = inputs.predictor_planted(2048, 128, 0.11, seed=2100)
        f["mask"] = np.repeat(f["predictor"]["hot"][None].astype(np.uint8), 128, axis=0)
        a = inputs.config3_attn()
        ffn_calls = 2
    elif name in ("opt1.3b_layer_hostw", "opt1.3b_layer_hostw_overlap"):
        # the shared-list layer with the FFN weights resident in pinned HOST memory (Sec. VII-B,
        # memory footprint): every call gathers the listed neuron blocks of W_up and W_down_t over
        # the host link, transposes them on the device and runs the FFN on the compact matrices
        f = inputs.ffn_bernoulli(8192, 2048, 8192, 64, 64, 0.11, seed=2100, dtype="bf16")
        f["predictor"] = inputs.predictor_planted(2048, 128, 0.11, seed=2100)
        f["mask"] = np.repeat(f["predictor"]["hot"][None].astype(np.uint8), 128, axis=0)
        f["host_weights"] = "overlap" if name.endswith("_overlap") else True
        a = inputs.config3_attn()
        ffn_calls = 2
    elif name == "opt1.3b_layer_lora":
        # the default layer with a LoRA branch (rank 16) on the FFN up-projection: forward, input
        # gradient and the gradients of the trainable A and B under the mask (Sec. II-C / II-D)
        f = inputs.ffn_planted_support(8192, 2048, 8192, 64, 64, 0.5, 4.0, seed=2000)
        f["lora"] = inputs.lora_matrices(2048, 8192, 16, seed=2200)
        a = inputs.config3_attn()
        ffn_calls = 2
    elif name == "opt1.3b_layer_f16":
        # the default layer in IEEE half precision (fp16 operands, fp32 accumulation): the
        # parameter precision of the paper's own runs (Sec. VII-A); same recipes and seeds
        f = inputs.ffn_planted_support(8192, 2048, 8192, 64, 64, 0.5, 4.0, seed=2000, dtype="f16")
        a = inputs.config3_attn(dtype="f16")
        ffn_calls = 2
    elif name == "opt1.3b_layer_patterns":
        # attention masks the way the paper forms them (Sec. VI-A): every head is assigned one
        # pattern of a pool whose layouts were computed beforehand; the step combines them into
        # the multi-head list on the device instead of compacting dense masks
        f = inputs.ffn_planted_support(8192, 2048, 8192, 64, 64, 0.5, 4.0, seed=2000)
        a = inputs.config3_patterns()
        ffn_calls = 2
    elif name == "config4":
        f = inputs.config4_ffn()
        a = inputs.config4_attn()
        ffn_calls = 1
    elif name.startswith("config5:"):
        parts = name.split(":")
        rho = float(parts[1])
        f = inputs.config5_ffn(rho)
        a = inputs.config5_attn(rho)
        ffn_calls = 1
        if len(parts) > 2 and parts[2] == "shared":
            # the same layer with ONE list row for all token tiles (row 0 of the mask, repeated), which
            # lets a workgroup take up to four token tiles: the dense path at rho = 1
            f["mask"] = np.repeat(f["mask"][:1], f["mask"].shape[0], axis=0)
            # four token tiles per workgroup asked for: measured faster at these shapes than the
            # library's own choice also where that leaves CUs without a workgroup (10 %: 128 items of
            # four tiles 0.71 ms per step, 256 items of two tiles 0.78 ms)
            f["shared_list"], f["tiles_per_wg"] = True, 4
    else:
        raise SystemExit(f"unknown workload {name!r}")
    return f, a, ffn_calls


class FfnJob:
    """One lx_sparse_ffn_fwd + lx_sparse_ffn_bwd_dx call pair on T tokens."""

    def __init__(self, lx, torch, f, rows, wsets):
        """wsets: list of (W_up, W_down, W_up_t, W_down_t) device copies of the frozen weights; a
        step uses set number self.wsel (one set: cache-warm; several rotated: cache-cold)."""
        from util import dev, lx_dtype
        self.lx, self.torch = lx, torch
        self.wsets, self.wsel = wsets, 0
        Wu, Wd, Wut, Wdt = wsets[0]
        sl = slice(rows[0] * 64, rows[1] * 64)
        self.dt = f["dtype"]
        self.X = dev(f["X"][sl], self.dt)
        self.dY = dev(f["dY"][sl], self.dt)
        self.mask_h = np.ascontiguousarray(f["mask"][rows[0]:rows[1]])
        self.T, self.d = self.X.shape
        self.F = Wu.shape[0]
        Tt, Fb = self.mask_h.shape
        self.nnz = int(self.mask_h.sum())          # active (tile, block) pairs
        self.pred = f.get("predictor")
        if self.pred is None and f.get("shared_list"):   # one input row for all token tiles
            assert (self.mask_h == self.mask_h[:1]).all()
            self.mask = torch.from_numpy(np.ascontiguousarray(self.mask_h[:1])).cuda()
            lrows, lnnz = 1, int(self.mask_h[0].sum())
        elif self.pred is None:                    # mask rows are inputs, one per token tile
            self.mask = torch.from_numpy(self.mask_h).cuda()
            lrows, lnnz = Tt, self.nnz
        else:                                      # one row, written by the predictor every step
            self.Wa_t = dev(self.pred["Wa_t"], self.dt)
            self.mask = torch.zeros((1, Fb), dtype=torch.uint8, device="cuda")
            lrows, lnnz = 1, int(self.pred["hot"].sum())
        self.cap = lrows * Fb
        self.bl = lx.BlockList(lrows, Fb, torch.empty(lrows + 1, dtype=torch.int32, device="cuda"),
                               torch.empty(self.cap, dtype=torch.int32, device="cuda"), self.cap)
        # H_act sized by the host-known active count (the mask is a host-generated input)
        self.bl_run = lx.BlockList(lrows, Fb, self.bl.row_ptr, self.bl.col_idx, max(lnnz, 1))
        self.H_act = torch.empty(max(self.nnz, 1) * 4096, dtype=self.X.dtype, device="cuda")
        self.Y = torch.empty_like(self.X)
        self.dX = torch.empty_like(self.X)
        nb = lx.lx_sparse_ffn_bwd_workspace_bytes(lx_dtype(lx, self.dt), self.T, self.d, self.F, 64, 64,
                                                  max(self.nnz, 1), 1)
        # extra workspace with which the second product of a pass splits the lists of its last
        # round of workgroups (one list row only; 0 bytes where the library would not split)
        extra = lx.lx_sparse_ffn_split_workspace_bytes(lx_dtype(lx, self.dt), self.T, self.d, 64, self.bl_run)
        self.ws = torch.empty(nb + extra, dtype=torch.uint8, device="cuda")
        self.ws_fwd = torch.empty(extra, dtype=torch.uint8, device="cuda") if extra else None
        self.used = float((self.mask_h.sum(0) > 0).mean())     # fraction of neuron blocks touched
        self.hostw = bool(f.get("host_weights"))
        self.gathered = False
        if self.hostw:
            # host copies of the two neuron-major matrices; device buffers for the listed blocks
            self.Wu_h, self.Wdt_h = Wu.cpu().pin_memory(), Wdt.cpu().pin_memory()
            cap = self.bl_run.nnz_cap
            mk = lambda r, c: torch.zeros((r, c), dtype=self.X.dtype, device="cuda")
            self.Wu_c, self.Wdt_c = mk(cap * 64, self.d), mk(cap * 64, self.d)
            self.Wd_c, self.Wut_c = mk(self.d, cap * 64), mk(self.d, cap * 64)
            self.cl = lx.BlockList(1, cap, torch.empty(2, dtype=torch.int32, device="cuda"),
                                   torch.empty(cap, dtype=torch.int32, device="cuda"), cap)
        self.lora = f.get("lora")
        if self.lora is not None:
            self.A_pad, self.B_pad = dev(self.lora["A_pad"], self.dt), dev(self.lora["B_pad"], self.dt)
            self.U = torch.empty((self.T, 64), dtype=self.X.dtype, device="cuda")
            self.dA = torch.empty((64, self.d), dtype=torch.float32, device="cuda")
            self.dB = torch.empty((self.F, 64), dtype=torch.float32, device="cuda")
            self.ws = torch.empty(lx.lx_sparse_ffn_lora_bwd_workspace_bytes(self.T, self.d, self.F,
                                                                            max(self.nnz, 1)),
                                  dtype=torch.uint8, device="cuda")
            self.ws_f = torch.empty(lx.lx_sparse_ffn_lora_fwd_workspace_bytes(self.T, self.d), dtype=torch.uint8,
                                    device="cuda")

    Wu = property(lambda self: self.wsets[self.wsel][0])
    Wd = property(lambda self: self.wsets[self.wsel][1])
    Wut = property(lambda self: self.wsets[self.wsel][2])
    Wdt = property(lambda self: self.wsets[self.wsel][3])

    def gather(self):
        """Host-resident weights: the listed blocks of both neuron-major matrices -> device, on the
        current stream."""
        lx = self.lx
        lx.lx_ffn_gather_weight_blocks(self.Wu_h, self.bl_run, 64, out=self.Wu_c, compact=self.cl)
        lx.lx_ffn_gather_weight_blocks(self.Wdt_h, self.bl_run, 64, out=self.Wdt_c, compact=self.cl)
        self.gathered = True

    def predict(self):
        if self.pred is not None:
            self.lx.lx_mlp_predict_mask(self.X, self.Wa_t, self.pred["thr"], self.T, mask=self.mask)

    def run(self):
        lx = self.lx
        if self.lora is not None:
            lx.lx_sparse_ffn_lora_fwd(self.X, self.Wu, self.A_pad, self.B_pad, self.Wd, self.bl_run,
                                      self.Y, self.H_act, self.U, self.ws_f)
            lx.lx_sparse_ffn_lora_bwd(self.X, self.dY, self.H_act, self.U, self.Wut, self.Wdt,
                                      self.A_pad, self.B_pad, self.bl_run, self.dX, self.dA, self.dB,
                                      self.ws)
            return
        if self.hostw:
            if not self.gathered:
                self.gather()
            self.gathered = False
            lx.lx_ffn_transpose(self.Wdt_c, out=self.Wd_c)
            lx.lx_ffn_transpose(self.Wu_c, out=self.Wut_c)
            lx.lx_sparse_ffn_fwd(self.X, self.Wu_c, self.Wd_c, self.cl, 64, 64, self.Y, self.H_act)
            lx.lx_sparse_ffn_bwd_dx(self.dY, self.H_act, self.Wu_c, self.Wd_c, self.cl, 64, 64, self.dX,
                                    self.ws, W_up_t=self.Wut_c, W_down_t=self.Wdt_c)
            return
        lx.lx_sparse_ffn_fwd(self.X, self.Wu, self.Wd, self.bl_run, 64, 64, self.Y, self.H_act,
                             workspace=self.ws_fwd)
        lx.lx_sparse_ffn_bwd_dx(self.dY, self.H_act, self.Wu, self.Wd, self.bl_run, 64, 64, self.dX,
                                self.ws, W_up_t=self.Wut, W_down_t=self.Wdt)

    def flops_per_gemm(self):
        return self.nnz * 2.0 * 64 * 64 * self.d

    def bytes_sdd(self):   # X (or dY) + touched weight blocks + compact activations written
        return 2.0 * (self.T * self.d + self.used * self.F * self.d + self.nnz * 4096)

    def bytes_dsd(self):   # compact activations read + touched weight blocks + Y (or dX)
        return 2.0 * (self.nnz * 4096 + self.used * self.F * self.d + self.T * self.d)


class AttnJob:
    def __init__(self, lx, torch, a):
        from util import dev, lx_dtype
        self.lx, self.torch, self.a = lx, torch, a
        self.Q, self.K, self.V, self.dO = (dev(a[k], a["dtype"]) for k in ("Q", "K", "V", "dO"))
        self.ha = torch.from_numpy(a["head_active"]).cuda()
        B, Hh, S, D = self.Q.shape
        self.B, self.Hh, self.S, self.D = B, Hh, S, D
        nb = S // 64
        mb = a["mask_batch"]
        self.pool = a.get("pool")
        if self.pool is None:                      # dense masks, compacted every step
            self.mask = torch.from_numpy(a["mask"]).cuda()
            blocks_per_head = a["mask"].sum(axis=(2, 3))                  # [mb, Hh]
        else:                                      # offline: the layouts of the pool's patterns
            self.pool_r, self.pool_c = lx.lx_mask_compact_pair(torch.from_numpy(self.pool).cuda())
            self.hp = torch.from_numpy(a["head_pattern"]).cuda()
            hp = a["head_pattern"].reshape(mb, Hh)
            blocks_per_head = np.where(hp >= 0, self.pool.sum(axis=(1, 2))[np.maximum(hp, 0)], 0)
        rows = mb * Hh * nb
        mk = lambda: lx.BlockList(rows, nb, torch.empty(rows + 1, dtype=torch.int32, device="cuda"),
                                  torch.empty(rows * nb, dtype=torch.int32, device="cuda"), rows * nb)
        self.bl_r, self.bl_c = mk(), mk()
        self.O = torch.empty_like(self.Q)
        self.LSE = torch.empty((B, Hh, S), dtype=torch.float32, device="cuda")
        self.dQ, self.dK, self.dV = (torch.empty_like(self.Q) for _ in range(3))
        self.ws = torch.empty(lx.lx_sparse_attn_bwd_workspace_bytes(lx_dtype(lx, a["dtype"]), B, Hh, S, D),
                              dtype=torch.uint8, device="cuda")
        act = a["head_active"].astype(bool)
        self.h_act = int(act.sum())
        per_batch = blocks_per_head[:, act].sum(axis=1)        # blocks per mask batch entry
        self.nblk = float(per_batch.sum() * (B if mb == 1 else 1))
        self.density = float(blocks_per_head.sum() / (mb * Hh * nb * (nb + 1) / 2))   # over all heads

    def combine(self):
        if self.pool is not None:
            self.lx.lx_attn_combine_patterns(self.pool_r, self.pool_c, self.S // 64, self.hp,
                                             out=(self.bl_r, self.bl_c))

    def run(self):
        lx, a = self.lx, self.a
        lx.lx_sparse_attn_fwd(self.Q, self.K, self.V, self.bl_r, a["scale"], a["causal"], self.O,
                              self.LSE, mask_batch=a["mask_batch"], head_active=self.ha)
        lx.lx_sparse_attn_bwd_dx(self.Q, self.K, self.V, self.O, self.LSE, self.dO, self.bl_r,
                                 self.bl_c, a["scale"], a["causal"], self.dQ, self.dK, self.dV,
                                 self.ws, mask_batch=a["mask_batch"], head_active=self.ha)

    def unit_bytes(self):      # one [B, active heads, S, D] bf16 tensor
        return 2.0 * self.B * self.h_act * self.S * self.D

    def flops(self, gemms):    # `gemms` 64x64xD products per active block
        return self.nblk * gemms * 2.0 * 64 * 64 * self.D


# ----------------------------------------------------------------------------
# algorithmic work per kernel launch (what the method must do)
# ----------------------------------------------------------------------------

def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` as measured with rocprofv3's FETCH_SIZE / WRITE_SIZE
    counters (two --pmc runs of this script, scaled as the table's header explains); read from
    the committed summary profiles/hbm_traffic_<workload>.txt, None if there is no entry.  Also
    returns the commit the table says it was measured at: a table older than the kernels is
    stale, and the bench line says which kernels the figure belongs to."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        f"hbm_traffic_{workload}.txt")
    commit, traffic = None, None
    try:
        with open(path) as fh:
            for line in fh:
                c = line.split()
                if line.startswith("# measured_at_commit:"):
                    commit = c[2]          # the kernels the table was measured on
                elif len(c) >= 5 and not line.startswith("#") and kernel in c[0].split("+"):
                    traffic = (float(c[1]) * float(c[2]) + float(c[3]) * float(c[4])) * 1024.0
    except (OSError, ValueError):
        pass
    return traffic, commit


def kernel_model(lx, ffn_jobs, attn):
    """kernel id -> (launches per step, flops per launch, bytes per launch)."""
    fj = ffn_jobs[0]
    fl = float(np.mean([j.flops_per_gemm() for j in ffn_jobs]))
    bs = float(np.mean([j.bytes_sdd() for j in ffn_jobs]))
    bd = float(np.mean([j.bytes_dsd() for j in ffn_jobs]))
    n = len(ffn_jobs)
    u = attn.unit_bytes()
    stat = 4.0 * attn.B * attn.Hh * attn.S
    return {
        lx.LX_K_FFN_UP: (n, fl, bs), lx.LX_K_FFN_DOWN: (n, fl, bd),
        lx.LX_K_FFN_DH: (n, fl, bs + 2.0 * fj.nnz * 4096), lx.LX_K_FFN_DX: (n, fl, bd),
        lx.LX_K_ATTN_FWD: (1, attn.flops(2), 4 * u + stat),
        lx.LX_K_ATTN_BWD_DQ: (1, attn.flops(3), 6 * u + 2 * stat),
        lx.LX_K_ATTN_BWD_DKV: (1, attn.flops(4), 6 * u + 2 * stat),
        lx.LX_K_COMPACT: (1, 0.0, 0.0),
        **({lx.LX_K_COMBINE: (1, 0.0, 0.0)} if attn.pool is not None else {}),
        # three bracketed groups per call: U = X A^T; G = dZ B; dB, dA
        **({lx.LX_K_LORA: (3 * n, 0.0, 0.0)} if fj.lora is not None else {}),
        **({lx.LX_K_PREDICT: (n, 2.0 * fj.T * fj.d * fj.mask_h.shape[1],
                              2.0 * (fj.T * fj.d + fj.mask_h.shape[1] * fj.d))}
           if fj.pred is not None else {}),
    }


def cpu_baseline(f, a, ffn_tiles=3, attn_heads=24):
    """The oracle as it stands, single thread, on a bounded sample of the same
    workload: the first `ffn_tiles` token tiles (forward + input gradient) and
    the first `attn_heads` active heads of batch entry 0 (forward + backward).
    Token rates of the two halves are combined the same way a layer would run
    them: seconds per token add up."""
    from oracle import lx_oracle as oracle
    from util import round_to
    sl = slice(0, ffn_tiles * 64)
    m = np.ascontiguousarray(f["mask"][:ffn_tiles])
    t0 = time.perf_counter()
    if "lora" in f:
        r, Ap, Bp = f["lora"]["r"], f["lora"]["A_pad"], f["lora"]["B_pad"]
        U, H, _ = oracle.ffn_lora_fwd(f["X"][sl], f["W_up"], Ap[:r], Bp[:, :r], f["W_down"], m, 64, 64)
        oracle.ffn_lora_bwd(f["X"][sl], f["dY"][sl], f["W_up"], Ap[:r], Bp[:, :r], f["W_down"], m,
                            round_to(H, f["dtype"]) > 0, U, 64, 64)
    else:
        H, _ = oracle.ffn_fwd(f["X"][sl], f["W_up"], f["W_down"], m, 64, 64)
        oracle.ffn_bwd_dx(f["dY"][sl], f["W_up"], f["W_down"], m, round_to(H, f["dtype"]) > 0, 64, 64)
    t_ffn = time.perf_counter() - t0
    heads = np.nonzero(a["head_active"])[0][:attn_heads]
    sub = {k: np.ascontiguousarray(a[k][0:1, heads]) for k in ("Q", "K", "V", "dO")}
    if "pool" in a:
        nb = a["S"] // 64
        dense = oracle.combine_patterns(a["pool"], a["head_pattern"]).reshape(-1, a["Hh"], nb, nb)
    else:
        dense = a["mask"]
    mk = np.ascontiguousarray(dense[0:1, heads])
    t0 = time.perf_counter()
    oracle.attn_fwd(sub["Q"], sub["K"], sub["V"], mk, a["scale"], a["causal"], None, a["blk"])
    oracle.attn_bwd(sub["Q"], sub["K"], sub["V"], sub["dO"], mk, a["scale"], a["causal"], None,
                    a["blk"])
    t_att = time.perf_counter() - t0
    s_per_tok_ffn = t_ffn / (ffn_tiles * 64)
    # attention: an inactive head costs nothing; scale per-head time to all active heads
    n_act = int(a["head_active"].sum())
    s_per_tok_att = (t_att / len(heads)) * n_act / a["S"]
    return {
        "value": 1.0 / (s_per_tok_ffn + s_per_tok_att), "unit": "tokens/s", "cores": 1,
        "kind": "oracle",
        "sample": (f"first {ffn_tiles} token tiles of the FFN input ({t_ffn:.1f} s) and first "
                   f"{len(heads)} active heads of batch entry 0 ({t_att:.1f} s), fwd+bwd, fp64, "
                   "1 thread; per-token times of the two halves added"),
    }


def measure_peaks(lx, torch):
    """What the chip sustains, measured once before the timed region with the library's probes
    (lx_probe_mfma_rate: an MFMA issue loop on registers; lx_probe_stream_copy: a 16-byte-per-lane
    copy of 512 MiB, twice the capacity of the cache behind the fabric), best of five launches
    each, timed with events on the launch stream."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    src.zero_()

    def best(fn):
        t = []
        for _ in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            work = fn()
            e1.record()
            e1.synchronize()
            t.append((e0.elapsed_time(e1) * 1e-3, work))
        sec, work = min(t[1:])
        return work / sec

    mfma = best(lambda: lx.lx_probe_mfma_rate(4000, sink))
    copy = best(lambda: lx.lx_probe_stream_copy(src, dst))
    del src, dst
    return {"mfma_bf16_tflops": mfma / 1e12, "stream_copy_gbs": copy / 1e9}


def run(workload: str, steps: int, warmup: int, with_cpu: bool, cache: str = "warm", peaks=None,
        two_streams: bool = False):
    import torch
    from paper_2510_15964_amd import lx
    from util import dev

    assert torch.cuda.is_available(), "bench.py needs a GPU (no fallback path)"
    torch.cuda.set_device(0)
    f, a, ffn_calls = make_workload(workload)
    lx.lx_ffn_set_token_tiles_per_workgroup(f.get("tiles_per_wg", 0))   # 0 = the library chooses
    Wu, Wd = dev(f["W_up"], f["dtype"]), dev(f["W_down"], f["dtype"])
    Wut, Wdt = lx.lx_ffn_pack_weights(Wu, Wd)            # one-time repack of frozen weights
    wsets = [(Wu, Wd, Wut, Wdt)]
    if cache == "cold":
        # rotate among copies of the frozen weights that together exceed the 256 MB of cache
        # behind the fabric (at least three), so that no step finds its weights there
        one = sum(t.numel() * t.element_size() for t in wsets[0])
        while len(wsets) < 3 or len(wsets) * one <= (256 << 20):
            wsets.append(tuple(t.clone() for t in wsets[0]))
    Tt = f["mask"].shape[0]
    per = Tt // ffn_calls
    ffn_jobs = [FfnJob(lx, torch, f, (i * per, (i + 1) * per), wsets) for i in range(ffn_calls)]
    attn = AttnJob(lx, torch, a)
    tokens = a["B"] * a["S"]
    assert tokens == f["T"], "FFN and attention halves cover the same tokens"

    # all masks of the step (FFN token-tile masks, attention row and column lists): one launch
    cb = lx.CompactBatch()
    for j in ffn_jobs:
        cb.add(j.mask, j.bl)
    if attn.pool is None:
        cb.add(attn.mask, attn.bl_r).add(attn.mask, attn.bl_c, transpose=True)

    # Host-resident weights: the gathers of a step need only its lists, use no LDS and are bound
    # by the host link, so they run on a second stream (default priority) under the attention
    # kernels, which then go first; each FFN call waits for its own gather.
    overlap = f.get("host_weights") == "overlap"
    if overlap:
        side = torch.cuda.Stream()
        ev_lists = torch.cuda.Event()
        ev_done = [torch.cuda.Event() for _ in ffn_jobs]
    counter = [0]

    def step():
        for j in ffn_jobs:
            j.wsel = counter[0] % len(wsets)
            j.predict()
        counter[0] += 1
        lx.lx_mask_compact_batch(cb)
        attn.combine()
        if overlap:
            main = torch.cuda.current_stream()
            ev_lists.record(main)
            with torch.cuda.stream(side):
                side.wait_event(ev_lists)
                for j, ev in zip(ffn_jobs, ev_done):
                    j.gather()
                    ev.record(side)
            attn.run()
            for j, ev in zip(ffn_jobs, ev_done):
                main.wait_event(ev)
                j.run()
            side.wait_stream(main)      # the next step's gathers overwrite what this step's kernels read
            return
        for j in ffn_jobs:
            j.run()
        attn.run()

    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()
    for j in ffn_jobs:        # the predicted mask is the planted one (accounting relies on it)
        if j.pred is not None:
            assert np.array_equal(j.mask.cpu().numpy()[0].astype(bool), j.pred["hot"])

    # per-kernel breakdown (untimed pre-pass, 3 steps per kernel)
    model = kernel_model(lx, ffn_jobs, attn)
    per_kernel = {}
    for kid, (launches, _, _) in model.items():
        lx.lx_profile_begin(kid, 3 * launches)
        for _ in range(3):
            step()
        torch.cuda.synchronize()
        ms, n = lx.lx_profile_end()
        per_kernel[kid] = (ms / 3.0, ms / max(n, 1))      # ms per step, ms per launch
    dom = max((k for k in per_kernel if k not in (lx.LX_K_COMPACT, lx.LX_K_COMBINE, lx.LX_K_LORA)),
              key=lambda k: per_kernel[k][0])

    # timed region: exactly `steps` steps, dominant kernel bracketed by events
    lx.lx_profile_begin(dom, steps * model[dom][0])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dom_ms, dom_n = lx.lx_profile_end()
    dom_avg_s = dom_ms / max(dom_n, 1) * 1e-3

    # spread of single steps: a second pass of `steps` steps, each bracketed by a pair of events on
    # the launch stream (outside the timed region above, whose figure is the mean)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step_ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)

    # The FFN and the attention half of the step read different inputs, so a caller may give them a
    # stream each (the lists first, then both halves side by side).  Reported next to the headline,
    # never as `value`: in a transformer layer the FFN consumes what attention produced.
    two_streams_ms = None
    if two_streams and not f.get("host_weights") and attn.pool is None and ffn_jobs[0].pred is None:
        side = torch.cuda.Stream()
        ev_lists, ev_attn = torch.cuda.Event(), torch.cuda.Event()

        def step_two_streams():
            for j in ffn_jobs:
                j.wsel = counter[0] % len(wsets)
            counter[0] += 1
            lx.lx_mask_compact_batch(cb)
            main = torch.cuda.current_stream()
            ev_lists.record(main)
            with torch.cuda.stream(side):
                side.wait_event(ev_lists)
                attn.run()
                ev_attn.record(side)
            for j in ffn_jobs:
                j.run()
            main.wait_event(ev_attn)

        for _ in range(3):
            step_two_streams()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            step_two_streams()
        torch.cuda.synchronize()
        two_streams_ms = (time.perf_counter() - t1) / steps * 1e3

    ms_per_step = elapsed / steps * 1e3
    flops_step = sum(model[k][0] * model[k][1] for k in model)
    _, fl, by = model[dom]
    t_mfma, t_hbm = fl / PEAK_MFMA_BF16, by / PEAK_HBM
    if t_mfma >= t_hbm:
        roof = {"bound": "mfma", "achieved": fl / dom_avg_s / 1e12, "peak": PEAK_MFMA_BF16 / 1e12,
                "unit": "TFLOP/s"}
        measured_peak = peaks["mfma_bf16_tflops"] if peaks else None
    else:
        roof = {"bound": "hbm", "achieved": by / dom_avg_s / 1e9, "peak": PEAK_HBM / 1e9,
                "unit": "GB/s"}
        measured_peak = peaks["stream_copy_gbs"] if peaks else None
    roof["frac"] = roof["achieved"] / roof["peak"]
    if measured_peak:
        roof["measured_peak"] = measured_peak            # the library's probe, same unit as `peak`
        roof["frac_of_measured"] = roof["achieved"] / measured_peak
    roof["traffic"], roof["traffic_measured_at_commit"] = measured_traffic(workload, lx.KERNEL_NAMES[dom])
    roof["algorithmic_bytes"] = by
    roof["kernel"] = lx.KERNEL_NAMES[dom]
    roof["avg_launch_us"] = dom_avg_s * 1e6
    roof["launches_timed"] = dom_n

    ffn_ms = sum(per_kernel[k][0] for k in (lx.LX_K_FFN_UP, lx.LX_K_FFN_DOWN, lx.LX_K_FFN_DH,
                                            lx.LX_K_FFN_DX))
    att_ms = sum(per_kernel[k][0] for k in (lx.LX_K_ATTN_FWD, lx.LX_K_ATTN_BWD_DQ,
                                            lx.LX_K_ATTN_BWD_DKV))
    ffn_fl = sum(model[k][0] * model[k][1] for k in (lx.LX_K_FFN_UP, lx.LX_K_FFN_DOWN,
                                                     lx.LX_K_FFN_DH, lx.LX_K_FFN_DX))
    att_fl = flops_step - ffn_fl
    out = {
        "metric": METRIC, "value": tokens * steps / elapsed, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": per_step_ms[len(per_step_ms) // 2], "ms_per_step_min": per_step_ms[0],
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": f["dtype"], "data": "synthetic",
        "cache": cache,
        "config": {
            "workload": workload, "tokens_per_step": tokens,
            "ffn": {"T_per_call": ffn_jobs[0].T, "calls": ffn_calls, "d": f["d"], "F": f["F"],
                    "block": "64x64", "block_density": float(f["mask"].mean()),
                    "active_blocks": int(f["mask"].sum()),
                    "list_rows_per_call": ffn_jobs[0].bl.rows,
                    "token_tiles_per_workgroup": f.get("tiles_per_wg", 0) or "auto",
                    "weight_sets": len(wsets),
                    "weight_bytes_all_sets": len(wsets) * sum(t.numel() * t.element_size() for t in wsets[0])},
            "attn": {"B": a["B"], "heads": a["Hh"], "active_heads": attn.h_act, "S": a["S"],
                     "D": a["D"], "causal": bool(a["causal"]),
                     "block_density_in_causal_region": attn.density,
                     "active_blocks": attn.nblk,
                     **({"mask_source": "pattern pool, combined on the device every step"}
                        if attn.pool is not None else {})},
        },
        "launches_per_step": int(sum(model[k][0] for k in model)),
        "active_tflops": flops_step / (elapsed / steps) / 1e12,
        "mfma_util_active_flops": flops_step / (elapsed / steps) / PEAK_MFMA_BF16,
        "ffn": {"ms_per_step_kernels": ffn_ms, "active_tflops": ffn_fl / (ffn_ms * 1e-3) / 1e12,
                "mfma_util": ffn_fl / (ffn_ms * 1e-3) / PEAK_MFMA_BF16},
        "attn": {"ms_per_step_kernels": att_ms, "active_tflops": att_fl / (att_ms * 1e-3) / 1e12,
                 "mfma_util": att_fl / (att_ms * 1e-3) / PEAK_MFMA_BF16},
        "kernels_us_per_launch": {lx.KERNEL_NAMES[k]: round(v[1] * 1e3, 2)
                                  for k, v in per_kernel.items()},
        "roofline": roof,
    }
    if peaks:
        out["measured_peaks"] = peaks
        out["mfma_util_active_flops_of_measured"] = (flops_step / (elapsed / steps) / 1e12
                                                     / peaks["mfma_bf16_tflops"])
    if two_streams_ms is not None:
        out["two_streams"] = {"ms_per_step": two_streams_ms, "value": tokens / (two_streams_ms * 1e-3),
                              "what": "attention calls on a second stream beside the FFN calls"}
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(f, a)
    lx.lx_ffn_set_token_tiles_per_workgroup(0)
    return out


def density_efficiency(results):
    """E(rho) = rho * t(dense) / t(rho) from whole-step times of configs[4] workloads (Sec. VII-C:
    operator time against density): `results` maps workload name -> ms per step.  Two references:
    the dense PATH (rho = 1 with one list for all token tiles and four token tiles per workgroup,
    what a dense layer would run) and the sparse kernels themselves at rho = 1."""
    dense_path = results.get("config5:1.0:shared")
    dense_lists = results.get("config5:1.0")
    out = {}
    for wl, ms in results.items():
        rho = float(wl.split(":")[1])
        e = {"ms_per_step": ms}
        if dense_path:
            e["E_vs_dense_path"] = rho * dense_path / ms
        if dense_lists:
            e["E_vs_per_tile_lists_at_100pct"] = rho * dense_lists / ms
        out[wl] = e
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    help="opt1.3b_layer (default) | opt1.3b_layer_twocalls | opt1.3b_layer_shared | "
                         "opt1.3b_layer_patterns | opt1.3b_layer_lora | opt1.3b_layer_f16 | "
                         "opt1.3b_layer_hostw | config4 | config5:RHO[:shared]")
    ap.add_argument("--cache", choices=("warm", "cold"), default="warm",
                    help="cold: every step uses another of several copies of the frozen weights "
                         "(more than 256 MB in total), so that none is found in cache")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the legs next to the headline: measured peaks, the cache-cold "
                         "variant and the density-efficiency runs of configs[4]")
    ap.add_argument("--sweep", metavar="FILE", default=None,
                    help="also run the configs[4] density sweep, one JSON line per density into FILE")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build is single-GPU; run with --gpus 1 "
                         "(token tiles and (batch, head) pairs are independent: the path "
                         "shards without communication)")
    if not os.path.exists(os.path.join(ROOT, "paper_2510_15964_amd", "liblx_sparse.so")):
        import __graft_entry__
        __graft_entry__.build()
    from oracle import build as oracle_build
    oracle_build.build(force=False)
    peaks = None
    if not args.no_extras:
        import torch
        from paper_2510_15964_amd import lx
        torch.cuda.set_device(0)
        peaks = measure_peaks(lx, torch)
        log(f"measured peaks: {peaks}")
    res = run(args.workload, args.steps, args.warmup, not args.no_cpu_baseline, args.cache, peaks,
              two_streams=not args.no_extras)
    if not args.no_extras:
        if args.cache == "warm":
            cold = run(args.workload, max(args.steps // 2, 5), 2, False, "cold", peaks)
            res["cache_cold"] = {k: cold[k] for k in ("value", "ms_per_step", "ms_per_step_median",
                                                      "ms_per_step_min")}
            res["cache_cold"]["weight_bytes_all_sets"] = cold["config"]["ffn"]["weight_bytes_all_sets"]
            res["cache_cold"]["roofline_frac"] = cold["roofline"]["frac"]
            log(f"cache-cold: {cold['ms_per_step']:.3f} ms/step")
        if args.workload == DEFAULT_WORKLOAD:
            # the same layer with the FFN as two calls of configs[1]'s own 4096 tokens
            two = run("opt1.3b_layer_twocalls", max(args.steps // 2, 5), 2, False, "warm", peaks)
            res["ffn_as_two_calls"] = {k: two[k] for k in ("value", "ms_per_step", "ms_per_step_median",
                                                          "launches_per_step")}
            res["ffn_as_two_calls"]["roofline"] = {k: two["roofline"][k] for k in ("kernel", "bound", "frac",
                                                                                  "avg_launch_us")}
            log(f"FFN as two calls of 4096 tokens: {two['ms_per_step']:.3f} ms/step")
        # density efficiency at the benchmark spec's 10 % and 30 % (configs[4] shapes), short runs
        ms = {}
        for wl in ("config5:1.0:shared", "config5:0.1", "config5:0.3", "config5:0.1:shared",
                   "config5:0.3:shared"):
            r = run(wl, 5, 2, False)
            ms[wl] = r["ms_per_step"]
            log(f"{wl}: {r['ms_per_step']:.3f} ms/step, FFN at {100 * r['ffn']['mfma_util']:.1f} % of the MFMA peak")
            if wl == "config5:1.0:shared":
                res["dense_path"] = {"workload": wl, "ms_per_step": r["ms_per_step"],
                                     "ffn_mfma_util": r["ffn"]["mfma_util"],
                                     "ffn_active_tflops": r["ffn"]["active_tflops"]}
        res["density_efficiency"] = density_efficiency(ms)
    if args.sweep:
        from paper_2510_15964_amd.inputs import DENSITY_SWEEP
        os.makedirs(os.path.dirname(os.path.abspath(args.sweep)), exist_ok=True)
        # the densities with independent lists per token tile, then the paper's operating
        # mode (one list per call for all its token tiles, Sec. V-A) at 10 %, 30 % and 100 %
        lines = {}
        for wl in [f"config5:{rho}" for rho in DENSITY_SWEEP] + [
                "config5:0.1:shared", "config5:0.3:shared", "config5:1.0:shared"]:
            r = run(wl, max(args.steps // 5, 5), 2, False, "warm", peaks)
            log(f"{wl}: {r['ms_per_step']:.3f} ms/step, {r['active_tflops']:.1f} active TFLOP/s")
            lines[wl] = r
        eff = density_efficiency({wl: r["ms_per_step"] for wl, r in lines.items()})
        with open(args.sweep, "w") as fh:
            for wl, r in lines.items():
                r["density_efficiency"] = eff[wl]
                fh.write(json.dumps(r) + "\n")
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
