"""Thin ctypes binding of the C-ABI library declared in include/lx.h.

Only argument marshalling happens here: torch tensors supply device pointers
and the current HIP stream; every step of the operators runs inside the
library's kernels.  Importing this module fails loudly when the library has
not been built (run `python paper_2510_15964_amd/build.py`); there is no CPU
or PyTorch fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblx_sparse.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first "
        "(python paper_2510_15964_amd/build.py). There is no fallback path.")

_lib = C.CDLL(LIB_PATH)

LX_OK, LX_ERR_INVALID_ARG, LX_ERR_UNSUPPORTED, LX_ERR_WORKSPACE, LX_ERR_RUNTIME = range(5)
LX_F32, LX_BF16, LX_F16 = 0, 1, 2

EXPORTS = (
    "lx_status_string", "lx_mask_compact", "lx_mask_compact_pair", "lx_mask_compact_batch", "lx_ffn_pack_weights",
    "lx_ffn_gather_weight_blocks",
    "lx_sparse_ffn_fwd_workspace_bytes", "lx_sparse_ffn_bwd_workspace_bytes",
    "lx_sparse_ffn_split_workspace_bytes",
    "lx_sparse_ffn_fwd", "lx_sparse_ffn_bwd_dx", "lx_sparse_attn_bwd_workspace_bytes",
    "lx_sparse_attn_fwd", "lx_sparse_attn_bwd_dx", "lx_sparse_attn_bwd_dx_noalloc", "lx_profile_begin", "lx_profile_end",
    "lx_attn_set_rows_per_workgroup", "lx_ffn_set_token_tiles_per_workgroup", "lx_mlp_predict_mask", "lx_attn_combine_patterns",
    "lx_sparse_ffn_lora_fwd_workspace_bytes", "lx_sparse_ffn_lora_bwd_workspace_bytes",
    "lx_sparse_ffn_lora_fwd", "lx_sparse_ffn_lora_bwd", "lx_probe_mfma_rate", "lx_probe_stream_copy",
)
(LX_K_COMPACT, LX_K_FFN_UP, LX_K_FFN_DOWN, LX_K_FFN_DH, LX_K_FFN_DX, LX_K_ATTN_FWD,
 LX_K_ATTN_BWD_DQ, LX_K_ATTN_BWD_DKV, LX_K_TRANSPOSE, LX_K_PREDICT, LX_K_COMBINE,
 LX_K_LORA) = range(12)
KERNEL_NAMES = ("compact", "ffn_up", "ffn_down", "ffn_dh", "ffn_dx", "attn_fwd", "attn_bwd_dq",
                "attn_bwd_dkv", "transpose", "predict", "combine", "lora")


class lx_blocklist(C.Structure):
    _fields_ = [("rows", C.c_int32), ("cols", C.c_int32), ("row_ptr", C.c_void_p),
                ("col_idx", C.c_void_p), ("nnz_cap", C.c_int32)]


_i32, _i64, _vp, _sz, _f = C.c_int32, C.c_int64, C.c_void_p, C.c_size_t, C.c_float


class lx_compact_job(C.Structure):
    _fields_ = [("mask", C.c_void_p), ("batch", C.c_int32), ("rows", C.c_int32),
                ("cols", C.c_int32), ("batch_stride", C.c_int64), ("row_stride", C.c_int64),
                ("col_stride", C.c_int64), ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p),
                ("col_idx_cap", C.c_int32)]
_blp = C.POINTER(lx_blocklist)
_lib.lx_status_string.restype = C.c_char_p
_lib.lx_status_string.argtypes = [C.c_int]
_lib.lx_mask_compact.argtypes = [_vp, _i32, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _i32, _vp]
_lib.lx_mask_compact_pair.argtypes = [_vp, _i32, _i32, _i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp,
                                      _i32, _vp]
_lib.lx_mask_compact_batch.argtypes = [C.POINTER(lx_compact_job), _i32, _vp]
_lib.lx_ffn_pack_weights.argtypes = [C.c_int, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
_lib.lx_ffn_gather_weight_blocks.argtypes = [C.c_int, _i32, _i32, _i32, _vp, _blp, _vp, _vp, _vp, _vp]
for _n in ("lx_sparse_ffn_fwd_workspace_bytes", "lx_sparse_ffn_bwd_workspace_bytes"):
    getattr(_lib, _n).restype = _sz
    getattr(_lib, _n).argtypes = [C.c_int, _i32, _i32, _i32, _i32, _i32, _i32, _i32]
_lib.lx_sparse_ffn_split_workspace_bytes.restype = _sz
_lib.lx_sparse_ffn_split_workspace_bytes.argtypes = [C.c_int, _i32, _i32, _i32, _blp]
_lib.lx_sparse_attn_bwd_workspace_bytes.restype = _sz
_lib.lx_sparse_attn_bwd_workspace_bytes.argtypes = [C.c_int, _i32, _i32, _i32, _i32]
_lib.lx_sparse_ffn_fwd.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp,
                                   _blp, _vp, _vp, _vp, _sz, _vp]
_lib.lx_sparse_ffn_bwd_dx.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp,
                                      _vp, _vp, _blp, _vp, _vp, _sz, _vp]
_lib.lx_sparse_attn_fwd.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _f, _i32, _vp, _vp, _vp,
                                    C.POINTER(_i64), _blp, _i32, _vp, _vp, _vp, _vp]
_lib.lx_sparse_attn_bwd_dx.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _f, _i32, _vp, _vp, _vp,
                                       _vp, _vp, _vp, C.POINTER(_i64), _blp, _blp, _i32, _vp, _vp,
                                       _vp, _vp, _vp, _sz, _vp]
_lib.lx_sparse_attn_bwd_dx_noalloc.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _f, _i32, _vp, _vp, _vp,
                                               _vp, _vp, _vp, C.POINTER(_i64), _blp, _blp, _i32, _vp,
                                               _vp, _vp, _vp, _vp]

_lib.lx_probe_mfma_rate.argtypes = [_i32, _vp, C.POINTER(C.c_double), _vp]
_lib.lx_probe_stream_copy.argtypes = [_vp, _vp, _sz, _vp]
_lib.lx_profile_begin.argtypes = [_i32, _i32]
_lib.lx_profile_end.argtypes = [C.POINTER(C.c_float), C.POINTER(_i32)]
_lib.lx_attn_set_rows_per_workgroup.argtypes = [_i32]
_lib.lx_ffn_set_token_tiles_per_workgroup.argtypes = [_i32]
_lib.lx_mlp_predict_mask.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _vp, _vp, _f, _vp, _vp]
_lib.lx_sparse_ffn_lora_fwd_workspace_bytes.restype = _sz
_lib.lx_sparse_ffn_lora_fwd_workspace_bytes.argtypes = [_i32, _i32]
_lib.lx_sparse_ffn_lora_bwd_workspace_bytes.restype = _sz
_lib.lx_sparse_ffn_lora_bwd_workspace_bytes.argtypes = [_i32, _i32, _i32, _i32]
_lib.lx_sparse_ffn_lora_fwd.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp,
                                        _blp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lx_sparse_ffn_lora_bwd.argtypes = [C.c_int, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp,
                                        _vp, _vp, _vp, _blp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.lx_attn_combine_patterns.argtypes = [_blp, _blp, _i32, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _i32,
                                          _vp]


class LxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_lib.lx_status_string(status).decode()}")


def status_string(status: int) -> str:
    return _lib.lx_status_string(status).decode()


def _check(status: int, where: str):
    if status != LX_OK:
        raise LxError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LX_F32
    if t.dtype == torch.bfloat16:
        return LX_BF16
    if t.dtype == torch.float16:
        return LX_F16
    raise LxError(LX_ERR_UNSUPPORTED, f"dtype {t.dtype}")


class BlockList:
    """Device-resident row-compressed active-block list plus its host header."""

    def __init__(self, rows: int, cols: int, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                 nnz_cap: int):
        self.rows, self.cols, self.nnz_cap = rows, cols, nnz_cap
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.c = lx_blocklist(rows, cols, row_ptr.data_ptr(), col_idx.data_ptr(), nnz_cap)


def lx_mask_compact(mask: torch.Tensor, transpose: bool = False, nnz_cap: int | None = None,
                    out: BlockList | None = None) -> BlockList:
    """mask: uint8 device tensor [..., R, C]; leading dims are flattened into
    the list's rows.  transpose=True builds the column-compressed list."""
    assert mask.dtype == torch.uint8 and mask.is_cuda and mask.is_contiguous() and mask.dim() >= 2
    R, Cc = mask.shape[-2], mask.shape[-1]
    batch = mask.numel() // (R * Cc)
    if transpose:
        rows, cols, rs, cs = Cc, R, 1, Cc
    else:
        rows, cols, rs, cs = R, Cc, Cc, 1
    cap = batch * rows * cols if nnz_cap is None else nnz_cap
    if out is None:
        row_ptr = torch.empty(batch * rows + 1, dtype=torch.int32, device=mask.device)
        col_idx = torch.empty(max(cap, 1), dtype=torch.int32, device=mask.device)
        out = BlockList(batch * rows, cols, row_ptr, col_idx, cap)
    _check(_lib.lx_mask_compact(_ptr(mask), batch, rows, cols, R * Cc, rs, cs, _ptr(out.row_ptr),
                                _ptr(out.col_idx), max(cap, 1), _stream()), "lx_mask_compact")
    return out


def lx_mask_compact_pair(mask: torch.Tensor, out=None):
    """Row list and column list of the same masks [..., R, C] in one launch."""
    assert mask.dtype == torch.uint8 and mask.is_cuda and mask.is_contiguous() and mask.dim() >= 2
    R, Cc = mask.shape[-2], mask.shape[-1]
    batch = mask.numel() // (R * Cc)
    cap = batch * R * Cc
    if out is None:
        mk = lambda rows, cols: BlockList(
            batch * rows, cols, torch.empty(batch * rows + 1, dtype=torch.int32, device=mask.device),
            torch.empty(cap, dtype=torch.int32, device=mask.device), cap)
        out = (mk(R, Cc), mk(Cc, R))
    blr, blc = out
    _check(_lib.lx_mask_compact_pair(_ptr(mask), batch, R, Cc, R * Cc, Cc, 1, _ptr(blr.row_ptr),
                                     _ptr(blr.col_idx), _ptr(blc.row_ptr), _ptr(blc.col_idx), cap,
                                     _stream()), "lx_mask_compact_pair")
    return blr, blc


class CompactBatch:
    """Pre-marshalled set of compaction jobs (up to 8) that run in one launch.
    add(mask, out, transpose) mirrors lx_mask_compact(mask, transpose, out=out)."""

    def __init__(self):
        self.jobs = []
        self._keep = []

    def add(self, mask: torch.Tensor, out: "BlockList", transpose: bool = False):
        assert mask.dtype == torch.uint8 and mask.is_cuda and mask.is_contiguous()
        R, Cc = mask.shape[-2], mask.shape[-1]
        batch = mask.numel() // (R * Cc)
        rows, cols, rs, cs = (Cc, R, 1, Cc) if transpose else (R, Cc, Cc, 1)
        assert out.rows == batch * rows and out.cols == cols
        self.jobs.append(lx_compact_job(mask.data_ptr(), batch, rows, cols, R * Cc, rs, cs,
                                        out.row_ptr.data_ptr(), out.col_idx.data_ptr(),
                                        out.col_idx.numel()))
        self._keep.append((mask, out))
        self._arr = (lx_compact_job * len(self.jobs))(*self.jobs)
        return self


def lx_mask_compact_batch(batch: CompactBatch):
    _check(_lib.lx_mask_compact_batch(batch._arr, len(batch.jobs), _stream()),
           "lx_mask_compact_batch")


def lx_attn_combine_patterns(pool_r: BlockList, pool_c: BlockList | None, nblk: int,
                             head_pattern: torch.Tensor, nnz_cap: int | None = None, out=None):
    """Multi-head list(s) from the pool layouts and the pattern id of every head.  Returns
    (row list, column list or None)."""
    assert head_pattern.dtype == torch.int32 and head_pattern.is_cuda and head_pattern.is_contiguous()
    Hm = head_pattern.numel()
    P = pool_r.rows // nblk
    cap = Hm * nblk * nblk if nnz_cap is None else nnz_cap
    if out is None:
        mk = lambda: BlockList(Hm * nblk, nblk,
                               torch.empty(Hm * nblk + 1, dtype=torch.int32, device=head_pattern.device),
                               torch.empty(max(cap, 1), dtype=torch.int32, device=head_pattern.device), cap)
        out = (mk(), mk() if pool_c is not None else None)
    blr, blc = out
    _check(_lib.lx_attn_combine_patterns(
        C.byref(pool_r.c), C.byref(pool_c.c) if pool_c is not None else None, P, nblk,
        _ptr(head_pattern), Hm, _ptr(blr.row_ptr), _ptr(blr.col_idx),
        _ptr(blc.row_ptr) if blc is not None else None, _ptr(blc.col_idx) if blc is not None else None,
        max(cap, 1), _stream()), "lx_attn_combine_patterns")
    return blr, blc


def lx_ffn_pack_weights(W_up: torch.Tensor, W_down: torch.Tensor):
    F, d = W_up.shape
    W_up_t = torch.empty((d, F), dtype=W_up.dtype, device=W_up.device)
    W_down_t = torch.empty((F, d), dtype=W_up.dtype, device=W_up.device)
    _check(_lib.lx_ffn_pack_weights(_dt(W_up), d, F, _ptr(W_up), _ptr(W_down), _ptr(W_up_t),
                                    _ptr(W_down_t), _stream()), "lx_ffn_pack_weights")
    return W_up_t, W_down_t


def lx_ffn_transpose(W: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """[R,C] -> [C,R] on the device (one half of lx_ffn_pack_weights)."""
    R, Cc = W.shape
    if out is None:
        out = torch.empty((Cc, R), dtype=W.dtype, device=W.device)
    assert out.shape == (Cc, R) and out.is_contiguous()
    _check(_lib.lx_ffn_pack_weights(_dt(W), Cc, R, _ptr(W), None, _ptr(out), None, _stream()),
           "lx_ffn_pack_weights")
    return out


def lx_ffn_gather_weight_blocks(W: torch.Tensor, bl: BlockList, blk_n: int, out=None, compact=None):
    """W [F,d]: device tensor or pinned host tensor; bl: one-row device list.  Returns
    (Wc [nnz_cap*blk_n, d] on the device, one-row list of the compact matrix)."""
    assert W.dim() == 2 and W.is_contiguous()
    F, d = W.shape
    dev = bl.row_ptr.device
    if out is None:
        out = torch.zeros((bl.nnz_cap * blk_n, d), dtype=W.dtype, device=dev)
    if compact is None:
        compact = BlockList(1, bl.nnz_cap, torch.empty(2, dtype=torch.int32, device=dev),
                            torch.empty(bl.nnz_cap, dtype=torch.int32, device=dev), bl.nnz_cap)
    _check(_lib.lx_ffn_gather_weight_blocks(_dt(W), d, F, blk_n, _ptr(W), C.byref(bl.c), _ptr(out),
                                            _ptr(compact.row_ptr), _ptr(compact.col_idx), _stream()),
           "lx_ffn_gather_weight_blocks")
    return out, compact


def lx_sparse_ffn_fwd_workspace_bytes(dt, T, d, F, tile_t, blk_n, nnz_cap, have_h_act) -> int:
    return _lib.lx_sparse_ffn_fwd_workspace_bytes(dt, T, d, F, tile_t, blk_n, nnz_cap, have_h_act)


def lx_sparse_ffn_bwd_workspace_bytes(dt, T, d, F, tile_t, blk_n, nnz_cap, have_packed) -> int:
    return _lib.lx_sparse_ffn_bwd_workspace_bytes(dt, T, d, F, tile_t, blk_n, nnz_cap, have_packed)


def lx_sparse_ffn_split_workspace_bytes(dt, T, d, tile_t, bl: "BlockList") -> int:
    return _lib.lx_sparse_ffn_split_workspace_bytes(dt, T, d, tile_t, C.byref(bl.c))


def lx_sparse_ffn_lora_fwd_workspace_bytes(T, d) -> int:
    return _lib.lx_sparse_ffn_lora_fwd_workspace_bytes(T, d)


def lx_sparse_ffn_lora_bwd_workspace_bytes(T, d, F, nnz_cap) -> int:
    return _lib.lx_sparse_ffn_lora_bwd_workspace_bytes(T, d, F, nnz_cap)


def lx_sparse_ffn_lora_fwd(X, W_up, A_pad, B_pad, W_down, bl: BlockList, Y, H_act, U, workspace=None):
    """U = X A_pad^T, H = ReLU(X W_up^T + U B_pad^T) on the listed blocks, Y = H W_down^T."""
    T, d = X.shape
    F = W_up.shape[0]
    assert A_pad.shape == (64, d) and B_pad.shape == (F, 64) and U.shape == (T, 64)
    if workspace is None:
        workspace = torch.empty(_lib.lx_sparse_ffn_lora_fwd_workspace_bytes(T, d), dtype=torch.uint8,
                                device=X.device)
    _check(_lib.lx_sparse_ffn_lora_fwd(_dt(X), T, d, F, 64, 64, _ptr(X), _ptr(W_up), _ptr(A_pad),
                                       _ptr(B_pad), _ptr(W_down), C.byref(bl.c), _ptr(Y), _ptr(H_act),
                                       _ptr(U), _ptr(workspace), workspace.numel(), _stream()),
           "lx_sparse_ffn_lora_fwd")


def lx_sparse_ffn_lora_bwd(X, dY, H_act, U, W_up_t, W_down_t, A_pad, B_pad, bl: BlockList, dX, dA, dB,
                           workspace):
    """dX, dA (fp32 [64,d]) and dB (fp32 [F,64]) of the LoRA-branch FFN."""
    T, d = X.shape
    F = W_down_t.shape[0]
    assert dA.dtype == torch.float32 and dA.shape == (64, d) and dB.dtype == torch.float32
    assert dB.shape == (F, 64) and W_up_t.shape == (d, F) and W_down_t.shape == (F, d)
    _check(_lib.lx_sparse_ffn_lora_bwd(_dt(X), T, d, F, 64, 64, _ptr(X), _ptr(dY), _ptr(H_act), _ptr(U),
                                       _ptr(W_up_t), _ptr(W_down_t), _ptr(A_pad), _ptr(B_pad),
                                       C.byref(bl.c), _ptr(dX), _ptr(dA), _ptr(dB), _ptr(workspace),
                                       workspace.numel(), _stream()), "lx_sparse_ffn_lora_bwd")


def lx_mlp_predict_mask(X: torch.Tensor, Wa_t: torch.Tensor, thr: float, group_rows: int,
                        mask: torch.Tensor | None = None):
    """mask [T/group_rows, nblk] uint8 = OR over the tokens of a group of (X Wa_t^T > thr)."""
    T, d = X.shape
    nblk = Wa_t.shape[0]
    assert Wa_t.shape == (nblk, d) and X.is_contiguous() and Wa_t.is_contiguous()
    if mask is None:
        mask = torch.empty((T // group_rows, nblk), dtype=torch.uint8, device=X.device)
    _check(_lib.lx_mlp_predict_mask(_dt(X), T, d, nblk, group_rows, _ptr(X), _ptr(Wa_t), thr,
                                    _ptr(mask), _stream()),
           "lx_mlp_predict_mask")
    return mask


def lx_sparse_attn_bwd_workspace_bytes(dt, B, Hh, S, D) -> int:
    return _lib.lx_sparse_attn_bwd_workspace_bytes(dt, B, Hh, S, D)


def lx_sparse_ffn_fwd(X, W_up, W_down, bl: BlockList, tile_t: int, blk_n: int, Y, H_act,
                      b_up=None, b_down=None, workspace=None):
    T, d = X.shape
    F = W_up.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.lx_sparse_ffn_fwd(_dt(X), T, d, F, tile_t, blk_n, _ptr(X), _ptr(W_up), _ptr(b_up),
                                  _ptr(W_down), _ptr(b_down), C.byref(bl.c), _ptr(Y), _ptr(H_act),
                                  _ptr(workspace), ws_bytes, _stream()), "lx_sparse_ffn_fwd")
    return Y


def lx_sparse_ffn_bwd_dx(dY, H_act, W_up, W_down, bl: BlockList, tile_t: int, blk_n: int, dX,
                         workspace, W_up_t=None, W_down_t=None):
    T, d = dY.shape
    F = W_up.shape[0] if W_up is not None else W_down_t.shape[0]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.lx_sparse_ffn_bwd_dx(_dt(dY), T, d, F, tile_t, blk_n, _ptr(dY), _ptr(H_act),
                                     _ptr(W_up), _ptr(W_down), _ptr(W_up_t), _ptr(W_down_t),
                                     C.byref(bl.c), _ptr(dX), _ptr(workspace), ws_bytes, _stream()),
           "lx_sparse_ffn_bwd_dx")
    return dX


def lx_profile_begin(kernel: int, max_launches: int):
    _check(_lib.lx_profile_begin(kernel, max_launches), "lx_profile_begin")


def lx_attn_set_rows_per_workgroup(rows: int):
    _check(_lib.lx_attn_set_rows_per_workgroup(rows), "lx_attn_set_rows_per_workgroup")


def lx_ffn_set_token_tiles_per_workgroup(tiles: int):
    _check(_lib.lx_ffn_set_token_tiles_per_workgroup(tiles), "lx_ffn_set_token_tiles_per_workgroup")


def lx_profile_end():
    """Returns (total kernel milliseconds, number of timed launches)."""
    ms, n = C.c_float(0), _i32(0)
    _check(_lib.lx_profile_end(C.byref(ms), C.byref(n)), "lx_profile_end")
    return ms.value, n.value


def _strides(t: torch.Tensor):
    assert t.dim() == 4 and t.stride(3) == 1
    return (_i64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def lx_sparse_attn_fwd(Q, K, V, bl: BlockList, scale: float, causal: bool, O, LSE,
                       mask_batch: int = 1, head_active=None):
    B, Hh, S, D = Q.shape
    for t in (K, V, O):
        assert t.stride() == Q.stride() and t.shape == Q.shape
    _check(_lib.lx_sparse_attn_fwd(_dt(Q), B, Hh, S, D, scale, int(causal), _ptr(Q), _ptr(K),
                                   _ptr(V), _strides(Q), C.byref(bl.c), mask_batch,
                                   _ptr(head_active), _ptr(O), _ptr(LSE), _stream()),
           "lx_sparse_attn_fwd")
    return O, LSE


def lx_sparse_attn_bwd_dx(Q, K, V, O, LSE, dO, bl_rows: BlockList, bl_cols: BlockList,
                          scale: float, causal: bool, dQ, dK, dV, workspace, mask_batch: int = 1,
                          head_active=None):
    B, Hh, S, D = Q.shape
    for t in (K, V, O, dO, dQ, dK, dV):
        assert t.stride() == Q.stride() and t.shape == Q.shape
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.lx_sparse_attn_bwd_dx(_dt(Q), B, Hh, S, D, scale, int(causal), _ptr(Q), _ptr(K),
                                      _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO), _strides(Q),
                                      C.byref(bl_rows.c), C.byref(bl_cols.c), mask_batch,
                                      _ptr(head_active), _ptr(dQ), _ptr(dK), _ptr(dV),
                                      _ptr(workspace), ws_bytes, _stream()),
           "lx_sparse_attn_bwd_dx")
    return dQ, dK, dV


def lx_sparse_attn_bwd_dx_noalloc(Q, K, V, O, LSE, dO, bl_rows: BlockList, bl_cols: BlockList,
                                  scale: float, causal: bool, dQ, dK, dV, mask_batch: int = 1,
                                  head_active=None):
    B, Hh, S, D = Q.shape
    for t in (K, V, O, dO, dQ, dK, dV):
        assert t.stride() == Q.stride() and t.shape == Q.shape
    _check(_lib.lx_sparse_attn_bwd_dx_noalloc(_dt(Q), B, Hh, S, D, scale, int(causal), _ptr(Q),
                                              _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO),
                                              _strides(Q), C.byref(bl_rows.c), C.byref(bl_cols.c),
                                              mask_batch, _ptr(head_active), _ptr(dQ), _ptr(dK),
                                              _ptr(dV), _stream()),
           "lx_sparse_attn_bwd_dx_noalloc")
    return dQ, dK, dV


def lx_probe_mfma_rate(iters: int, sink: torch.Tensor) -> float:
    """Enqueues the MFMA rate probe; returns the FLOP of the launch."""
    fl = C.c_double(0.0)
    _check(_lib.lx_probe_mfma_rate(iters, _ptr(sink), C.byref(fl), _stream()), "lx_probe_mfma_rate")
    return fl.value


def lx_probe_stream_copy(src: torch.Tensor, dst: torch.Tensor) -> int:
    """Enqueues the stream-copy probe; returns the bytes moved (read + written)."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check(_lib.lx_probe_stream_copy(_ptr(src), _ptr(dst), n, _stream()), "lx_probe_stream_copy")
    return 2 * n
