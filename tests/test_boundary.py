"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol that include/lx.h declares, and rejects bad arguments before any
launch."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lxmod():
    lib = os.path.join(ROOT, "paper_2510_15964_amd", "liblx_sparse.so")
    if not os.path.exists(lib):
        from paper_2510_15964_amd import build
        build.build()
    from paper_2510_15964_amd import lx
    return lx


def test_exports_every_declared_symbol(lxmod):
    hdr = open(os.path.join(ROOT, "include", "lx.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(lx_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(lxmod.EXPORTS)
    for name in declared:
        assert hasattr(lxmod._lib, name), name


def test_status_strings(lxmod):
    assert [lxmod.status_string(i) for i in range(5)] == [
        "LX_OK", "LX_ERR_INVALID_ARG", "LX_ERR_UNSUPPORTED", "LX_ERR_WORKSPACE", "LX_ERR_RUNTIME"]


FAKE = C.c_void_p(0x1000)      # non-null, 16-byte aligned, never dereferenced on these paths


def _bl(lxmod, rows, cols, cap=None):
    return lxmod.lx_blocklist(rows, cols, 0x1000, 0x1000, rows * cols if cap is None else cap)


def test_compact_rejects_bad_arguments(lxmod):
    f = lxmod._lib.lx_mask_compact
    assert f(None, 1, 4, 4, 16, 4, 1, FAKE, FAKE, 16, None) == lxmod.LX_ERR_INVALID_ARG
    assert f(FAKE, 1, 0, 4, 16, 4, 1, FAKE, FAKE, 16, None) == lxmod.LX_ERR_INVALID_ARG
    assert f(FAKE, 1, 4, 4, 16, 4, 1, FAKE, FAKE, 0, None) == lxmod.LX_ERR_INVALID_ARG
    assert f(FAKE, 1, 4, 4, 16, -4, 1, FAKE, FAKE, 16, None) == lxmod.LX_ERR_INVALID_ARG


def test_compact_pair_rejects_bad_arguments(lxmod):
    f = lxmod._lib.lx_mask_compact_pair
    assert f(FAKE, 1, 4, 4, 16, 4, 1, FAKE, FAKE, FAKE, None, 16, None) == lxmod.LX_ERR_INVALID_ARG
    assert f(FAKE, 1, 4, 0, 16, 4, 1, FAKE, FAKE, FAKE, FAKE, 16, None) == lxmod.LX_ERR_INVALID_ARG


def test_compact_batch_rejects_bad_arguments(lxmod):
    f = lxmod._lib.lx_mask_compact_batch
    J = lxmod.lx_compact_job
    ok = J(0x1000, 1, 4, 4, 16, 4, 1, 0x1000, 0x1000, 16)
    arr = (J * 2)(ok, J(0x1000, 1, 4, 4, 16, 4, 1, 0, 0x1000, 16))
    assert f(arr, 2, None) == lxmod.LX_ERR_INVALID_ARG          # second job has a null row_ptr
    assert f(arr, 0, None) == lxmod.LX_ERR_INVALID_ARG
    assert f(arr, 9, None) == lxmod.LX_ERR_INVALID_ARG
    assert f(None, 1, None) == lxmod.LX_ERR_INVALID_ARG


def _ffn_fwd(lxmod, dt, T, d, F, tt, bn, bl, X=FAKE, ws=None, ws_bytes=0, H=FAKE):
    return lxmod._lib.lx_sparse_ffn_fwd(dt, T, d, F, tt, bn, X, FAKE, None, FAKE, None,
                                        C.byref(bl) if bl is not None else None, FAKE, H, ws,
                                        ws_bytes, None)


def test_ffn_fwd_validation(lxmod):
    L = lxmod
    ok_bl = _bl(L, 8, 16)
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, ok_bl, X=None) == L.LX_ERR_INVALID_ARG
    assert _ffn_fwd(L, L.LX_BF16, 0, 128, 1024, 64, 64, ok_bl) == L.LX_ERR_INVALID_ARG
    assert _ffn_fwd(L, 7, 512, 128, 1024, 64, 64, ok_bl) == L.LX_ERR_UNSUPPORTED
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 32, 32, _bl(L, 16, 32)) == L.LX_ERR_UNSUPPORTED
    assert _ffn_fwd(L, L.LX_BF16, 512, 100, 1024, 64, 64, ok_bl) == L.LX_ERR_UNSUPPORTED
    assert _ffn_fwd(L, L.LX_BF16, 500, 128, 1024, 64, 64, ok_bl) == L.LX_ERR_UNSUPPORTED
    assert _ffn_fwd(L, L.LX_F32, 512, 128, 1024, 48, 48, ok_bl) == L.LX_ERR_UNSUPPORTED
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, None) == L.LX_ERR_INVALID_ARG
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, _bl(L, 8, 15)) == L.LX_ERR_INVALID_ARG
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, _bl(L, 8, 16, 999)) == L.LX_ERR_INVALID_ARG
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, ok_bl,
                    X=C.c_void_p(0x1004)) == L.LX_ERR_INVALID_ARG
    # no H_act buffer and no / too small workspace
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, ok_bl, H=None) == L.LX_ERR_WORKSPACE
    need = L.lx_sparse_ffn_fwd_workspace_bytes(L.LX_BF16, 512, 128, 1024, 64, 64, 128, 0)
    assert need >= 128 * 64 * 64 * 2
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, ok_bl, H=None, ws=FAKE,
                    ws_bytes=need - 1) == L.LX_ERR_WORKSPACE
    assert L.lx_sparse_ffn_fwd_workspace_bytes(L.LX_BF16, 512, 128, 1024, 64, 64, 128, 1) == 0


def test_ffn_bwd_validation(lxmod):
    L = lxmod
    bl = _bl(L, 8, 16)
    f = L._lib.lx_sparse_ffn_bwd_dx
    args = lambda **k: [k.get("dt", L.LX_BF16), 512, 128, 1024, 64, 64, k.get("dY", FAKE), FAKE,
                        k.get("Wu", FAKE), FAKE, k.get("Wut", FAKE), k.get("Wdt", FAKE),
                        C.byref(bl), FAKE, k.get("ws", FAKE), k.get("wsb", 1 << 30), None]
    assert f(*args(dY=None)) == L.LX_ERR_INVALID_ARG
    assert f(*args(Wut=None)) == L.LX_ERR_INVALID_ARG          # only one packed pointer
    assert f(*args(wsb=16)) == L.LX_ERR_WORKSPACE
    assert f(*args(ws=None)) == L.LX_ERR_WORKSPACE
    packed = L.lx_sparse_ffn_bwd_workspace_bytes(L.LX_BF16, 512, 128, 1024, 64, 64, 128, 1)
    raw = L.lx_sparse_ffn_bwd_workspace_bytes(L.LX_BF16, 512, 128, 1024, 64, 64, 128, 0)
    assert raw >= packed + 2 * 128 * 1024 * 2
    assert f(*args(Wut=None, Wdt=None, wsb=packed)) == L.LX_ERR_WORKSPACE


def test_attn_validation(lxmod):
    L = lxmod
    f = L._lib.lx_sparse_attn_fwd
    st = (C.c_int64 * 3)(32 * 256 * 64, 256 * 64, 64)
    bl = _bl(L, 32 * 4, 4)

    def call(dt=L.LX_BF16, B=2, Hh=32, S=256, D=64, strides=st, blist=bl, mb=1, Q=FAKE):
        return f(dt, B, Hh, S, D, 0.125, 1, Q, FAKE, FAKE, strides, C.byref(blist), mb, None, FAKE,
                 FAKE, None)

    assert call(dt=7) == L.LX_ERR_UNSUPPORTED            # no such element type
    assert call(dt=L.LX_F32, D=96) == L.LX_ERR_UNSUPPORTED
    assert call(D=96) == L.LX_ERR_UNSUPPORTED
    assert call(S=250) == L.LX_ERR_UNSUPPORTED
    assert call(Q=None) == L.LX_ERR_INVALID_ARG
    assert call(mb=3) == L.LX_ERR_INVALID_ARG
    assert call(blist=_bl(L, 32 * 4 - 1, 4)) == L.LX_ERR_INVALID_ARG
    assert call(strides=(C.c_int64 * 3)(32 * 256 * 64, 256 * 64, 60)) == L.LX_ERR_INVALID_ARG
    assert call(strides=None) == L.LX_ERR_INVALID_ARG
    g = L._lib.lx_sparse_attn_bwd_dx
    need = L.lx_sparse_attn_bwd_workspace_bytes(L.LX_BF16, 2, 32, 256, 64)
    assert need >= 2 * 32 * 256 * 4
    r = g(L.LX_BF16, 2, 32, 256, 64, 0.125, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, st, C.byref(bl),
          C.byref(bl), 1, None, FAKE, FAKE, FAKE, FAKE, need - 1, None)
    assert r == L.LX_ERR_WORKSPACE
    r = g(L.LX_BF16, 2, 32, 256, 64, 0.125, 1, FAKE, FAKE, FAKE, FAKE, None, FAKE, st, C.byref(bl),
          C.byref(bl), 1, None, FAKE, FAKE, FAKE, FAKE, need, None)
    assert r == L.LX_ERR_INVALID_ARG


def test_ffn_list_rows_must_divide_the_token_tiles(lxmod):
    L = lxmod
    # 8 token tiles: lists with 1, 2, 4, 8 rows are accepted by the validation (the H_act-less
    # call then fails on the workspace, after the list has been accepted), 3 rows are not
    for rows in (1, 2, 4, 8):
        assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, _bl(L, rows, 16), H=None) == \
            L.LX_ERR_WORKSPACE
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, _bl(L, 3, 16)) == L.LX_ERR_INVALID_ARG
    assert _ffn_fwd(L, L.LX_BF16, 512, 128, 1024, 64, 64, _bl(L, 16, 16)) == L.LX_ERR_INVALID_ARG


def test_gather_weight_blocks_validation(lxmod):
    """Everything that can be wrong with the sizes, the list and the pointers' alignment is found
    before the source pointer is looked at (and before any launch)."""
    L = lxmod
    f = L._lib.lx_ffn_gather_weight_blocks
    def call(dt=L.LX_BF16, d=128, F=512, blk=64, W=FAKE, bl=None, Wc=FAKE):
        bl = _bl(L, 1, F // blk if blk > 0 and F > 0 else 1) if bl is None else bl
        return f(dt, d, F, blk, W, C.byref(bl), Wc, None, None, None)
    assert call(dt=7) == L.LX_ERR_UNSUPPORTED
    assert call(d=0) == L.LX_ERR_INVALID_ARG
    assert call(F=500) == L.LX_ERR_INVALID_ARG                          # not whole neuron blocks
    assert call(blk=0) == L.LX_ERR_INVALID_ARG
    assert call(W=None) == L.LX_ERR_INVALID_ARG
    assert call(Wc=None) == L.LX_ERR_INVALID_ARG
    assert call(bl=_bl(L, 2, 8)) == L.LX_ERR_INVALID_ARG                # more than one list row
    assert call(bl=_bl(L, 1, 9)) == L.LX_ERR_INVALID_ARG                # columns are not F / blk_n
    assert call(bl=_bl(L, 1, 8, cap=0)) == L.LX_ERR_INVALID_ARG
    assert call(W=C.c_void_p(0x1008)) == L.LX_ERR_INVALID_ARG           # not 16-byte aligned
    assert call(dt=L.LX_F32, d=2, blk=1, F=8) == L.LX_ERR_INVALID_ARG   # a block is not whole 16-byte words


def test_mlp_predict_validation(lxmod):
    L = lxmod
    f = L._lib.lx_mlp_predict_mask
    args = lambda **k: [k.get("dt", L.LX_BF16), k.get("T", 512), k.get("d", 128), k.get("nblk", 128),
                        k.get("g", 512), k.get("X", FAKE), FAKE, k.get("thr", 1.0),
                        k.get("mask", FAKE), None]
    assert f(*args(dt=L.LX_F32)) == L.LX_ERR_UNSUPPORTED
    assert f(*args(T=500)) == L.LX_ERR_UNSUPPORTED
    assert f(*args(d=100)) == L.LX_ERR_UNSUPPORTED
    assert f(*args(nblk=100)) == L.LX_ERR_UNSUPPORTED
    assert f(*args(g=96)) == L.LX_ERR_INVALID_ARG              # not a multiple of 64
    assert f(*args(g=192)) == L.LX_ERR_INVALID_ARG             # does not divide T
    assert f(*args(X=None)) == L.LX_ERR_INVALID_ARG
    assert f(*args(mask=None)) == L.LX_ERR_INVALID_ARG
    assert f(*args(thr=float("nan"))) == L.LX_ERR_INVALID_ARG


def test_attn_combine_patterns_validation(lxmod):
    L = lxmod
    f = L._lib.lx_attn_combine_patterns
    pool = _bl(L, 8 * 16, 16)
    ok = lambda **k: [C.byref(k.get("pr", pool)) if k.get("pr", pool) is not None else None,
                      C.byref(k["pc"]) if k.get("pc") is not None else None,
                      k.get("P", 8), k.get("nblk", 16), k.get("hp", FAKE), k.get("H", 32),
                      k.get("rp", FAKE), k.get("ci", FAKE), k.get("rpc"), k.get("cic"),
                      k.get("cap", 1024), None]
    assert f(*ok(pr=None)) == L.LX_ERR_INVALID_ARG
    assert f(*ok(hp=None)) == L.LX_ERR_INVALID_ARG
    assert f(*ok(rp=None)) == L.LX_ERR_INVALID_ARG
    assert f(*ok(ci=None)) == L.LX_ERR_INVALID_ARG
    assert f(*ok(P=0)) == L.LX_ERR_INVALID_ARG
    assert f(*ok(H=0)) == L.LX_ERR_INVALID_ARG
    assert f(*ok(cap=0)) == L.LX_ERR_INVALID_ARG
    assert f(*ok(P=7)) == L.LX_ERR_INVALID_ARG                 # pool rows != P * nblk
    assert f(*ok(nblk=8)) == L.LX_ERR_INVALID_ARG              # pool cols != nblk
    assert f(*ok(pc=pool)) == L.LX_ERR_INVALID_ARG             # column pool without column outputs
    assert f(*ok(rpc=FAKE, cic=FAKE)) == L.LX_ERR_INVALID_ARG  # column outputs without a pool


def test_ffn_lora_validation(lxmod):
    L = lxmod
    bl = _bl(L, 8, 16)
    T, d, F = 512, 128, 1024

    def fwd(**k):
        need = L.lx_sparse_ffn_lora_fwd_workspace_bytes(k.get("T", T), k.get("d", d))
        b = k.get("bl", bl)
        return L._lib.lx_sparse_ffn_lora_fwd(
            k.get("dt", L.LX_BF16), k.get("T", T), k.get("d", d), k.get("F", F), k.get("tt", 64), 64,
            k.get("X", FAKE), FAKE, k.get("A", FAKE), FAKE, FAKE, C.byref(b) if b is not None else None,
            FAKE, k.get("H", FAKE), k.get("U", FAKE), k.get("ws", FAKE), k.get("wsb", need), None)

    def bwd(**k):
        need = L.lx_sparse_ffn_lora_bwd_workspace_bytes(T, d, F, bl.nnz_cap)
        b = k.get("bl", bl)
        return L._lib.lx_sparse_ffn_lora_bwd(
            k.get("dt", L.LX_BF16), k.get("T", T), d, F, 64, 64, k.get("X", FAKE), FAKE, FAKE,
            k.get("U", FAKE), k.get("Wut", FAKE), FAKE, FAKE, FAKE,
            C.byref(b) if b is not None else None, FAKE, k.get("dA", FAKE), k.get("dB", FAKE),
            k.get("ws", FAKE), k.get("wsb", need), None)

    for f in (fwd, bwd):
        assert f(dt=L.LX_F32) == L.LX_ERR_UNSUPPORTED            # bf16 only
        assert f(T=500) == L.LX_ERR_UNSUPPORTED
        assert f(X=None) == L.LX_ERR_INVALID_ARG
        assert f(U=None) == L.LX_ERR_INVALID_ARG
        assert f(bl=None) == L.LX_ERR_INVALID_ARG
        assert f(bl=_bl(L, 8, 15)) == L.LX_ERR_INVALID_ARG
        assert f(bl=_bl(L, 3, 16)) == L.LX_ERR_INVALID_ARG       # 8 tiles, 3 list rows
        assert f(ws=None) == L.LX_ERR_WORKSPACE
        assert f(X=C.c_void_p(0x1004)) == L.LX_ERR_INVALID_ARG
    assert fwd(tt=32) == L.LX_ERR_UNSUPPORTED
    assert fwd(d=100) == L.LX_ERR_UNSUPPORTED
    assert fwd(A=None) == L.LX_ERR_INVALID_ARG
    assert fwd(H=None) == L.LX_ERR_INVALID_ARG                   # the backward call needs it
    assert fwd(wsb=L.lx_sparse_ffn_lora_fwd_workspace_bytes(T, d) - 1) == L.LX_ERR_WORKSPACE
    assert bwd(Wut=None) == L.LX_ERR_INVALID_ARG                 # packed transposes are required
    assert bwd(dA=None) == L.LX_ERR_INVALID_ARG
    assert bwd(dB=None) == L.LX_ERR_INVALID_ARG
    assert bwd(wsb=L.lx_sparse_ffn_lora_bwd_workspace_bytes(T, d, F, bl.nnz_cap) - 1) == L.LX_ERR_WORKSPACE
    # sizes: the K split of U needs T*64 floats per range; degenerate shapes give the fixed minimum
    assert L.lx_sparse_ffn_lora_fwd_workspace_bytes(4096, 2048) >= 4 * 4096 * 64 * 4
    assert L.lx_sparse_ffn_lora_fwd_workspace_bytes(0, 0) == 256
    assert L.lx_sparse_ffn_lora_bwd_workspace_bytes(0, 128, 1024, 16) == 0
    assert (L.lx_sparse_ffn_lora_bwd_workspace_bytes(T, d, F, 128)
            >= 128 * 8192 + 64 * F * 2 + d * 64 * 2 + T * 64 * 2)


def test_half_precision_is_accepted_where_bfloat16_is(lxmod):
    """LX_F16 passes the dtype check of every 16-bit entry point (the next check then fails on
    the deliberately bad argument); unknown dtype codes and fp32 where it is not built do not."""
    L = lxmod
    bl = _bl(L, 8, 16)
    for dt in (L.LX_BF16, L.LX_F16):
        assert _ffn_fwd(L, dt, 512, 128, 1024, 64, 64, bl, X=None) == L.LX_ERR_INVALID_ARG
        assert _ffn_fwd(L, dt, 512, 128, 1024, 32, 32, _bl(L, 16, 32)) == L.LX_ERR_UNSUPPORTED
        assert L._lib.lx_mlp_predict_mask(dt, 512, 128, 128, 512, None, FAKE, 1.0, FAKE,
                                          None) == L.LX_ERR_INVALID_ARG
        assert L._lib.lx_sparse_ffn_lora_fwd(dt, 512, 128, 1024, 64, 64, None, FAKE, FAKE, FAKE, FAKE,
                                             C.byref(bl), FAKE, FAKE, FAKE, FAKE, 1 << 30,
                                             None) == L.LX_ERR_INVALID_ARG
        assert L.lx_sparse_ffn_bwd_workspace_bytes(dt, 512, 128, 1024, 64, 64, 128, 1) == 128 * 8192
    assert _ffn_fwd(L, 3, 512, 128, 1024, 64, 64, bl) == L.LX_ERR_UNSUPPORTED
    assert L._lib.lx_mlp_predict_mask(L.LX_F32, 512, 128, 128, 512, FAKE, FAKE, 1.0, FAKE,
                                      None) == L.LX_ERR_UNSUPPORTED


def test_tuning_knobs_reject_values_outside_their_range(lxmod):
    L = lxmod
    for v in (3, 5, 8, -1):
        assert L._lib.lx_ffn_set_token_tiles_per_workgroup(v) == L.LX_ERR_INVALID_ARG
    for v in (4, 2, 1, 0):
        assert L._lib.lx_ffn_set_token_tiles_per_workgroup(v) == L.LX_OK
    assert L._lib.lx_attn_set_rows_per_workgroup(9) == L.LX_ERR_INVALID_ARG
    assert L._lib.lx_attn_set_rows_per_workgroup(0) == L.LX_OK
