"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes its buffers as documented and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2012_02030_amd import binding as ap

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(ap.LIB_PATH):
        from paper_2012_02030_amd import build
        build.build()
    return ap.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ap_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert set(ap.SYMBOLS) == set(names)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings(L):
    assert ap.ap_status_string(0) == "AP_OK"
    assert ap.ap_status_string(-1) == "AP_ERR_INVALID_ARG"
    assert ap.ap_status_string(-2) == "AP_ERR_UNSUPPORTED"
    assert ap.ap_status_string(-3) == "AP_ERR_CAPACITY"
    assert ap.ap_status_string(-4) == "AP_ERR_HIP"


def test_layout_sizes(L):
    assert ap.ap_layout_max_tiles(16, 4096, 4096, 64, 64) == 16 * 64 * 64
    assert ap.ap_layout_max_tiles(2, 65, 130, 64, 64) == 2 * 2 * 3
    assert ap.ap_layout_max_tiles(1, 64, 64, 48, 64) == -1          # unsupported block size
    assert ap.ap_layout_max_tiles(0, 64, 64, 64, 64) == -1
    ws = ap.ap_layout_workspace_bytes(16, 4096, 4096, 64, 64)
    tiles = 16 * 64 * 64
    assert ws >= tiles * 64 * 8 + tiles + 16 * 64 * 4                # dense bitmaps + flags + counts
    assert ws < 1.1 * (tiles * 64 * 8 + tiles + 16 * 64 * 4) + 64
    assert ap.ap_layout_workspace_bytes(1, 64, 64, 48, 64) == 0


def test_build_layout_rejects_bad_arguments(L):
    fake = 0x1000   # never dereferenced: validation fails first
    call = L.ap_build_layout
    ok_ws = ap.ap_layout_workspace_bytes(2, 64, 64, 64, 64)
    assert call(None, 2, 64, 64, 64, 64, fake, fake, fake, 8, fake, fake, ok_ws, None) == ap.AP_ERR_INVALID_ARG
    assert call(fake, 0, 64, 64, 64, 64, fake, fake, fake, 8, fake, fake, ok_ws, None) == ap.AP_ERR_INVALID_ARG
    assert call(fake, 2, 64, 64, 48, 64, fake, fake, fake, 8, fake, fake, ok_ws, None) == ap.AP_ERR_UNSUPPORTED
    assert call(fake, 2, 64, 64, 64, 64, fake, fake, None, 8, fake, fake, ok_ws, None) == ap.AP_ERR_INVALID_ARG
    assert call(fake, 2, 64, 64, 64, 64, fake, fake, fake, -1, fake, fake, ok_ws, None) == ap.AP_ERR_INVALID_ARG
    assert call(fake, 2, 64, 64, 64, 64, fake, fake, fake + 4, 8, fake, fake, ok_ws, None) == ap.AP_ERR_INVALID_ARG
    assert call(fake, 2, 64, 64, 64, 64, fake, fake, fake, 8, fake, fake, ok_ws - 1, None) == ap.AP_ERR_CAPACITY
    assert call(fake, 2, 64, 64, 64, 64, fake, fake, fake, 8, fake, None, ok_ws, None) == ap.AP_ERR_INVALID_ARG


def _fwd(L, **over):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)
    a = dict(Q=fake, K=fake + 0x100000, V=fake + 0x200000, O=fake + 0x300000, lse=None, dtype=ap.AP_BF16,
             B=1, H=2, Lq=64, Lk=64, D=64, sq=s, sk=s, sv=s, so=s, row_ptr=fake, col_idx=fake,
             bitmaps=fake, bm=64, bn=64, causal=0, scale=0.0)
    a.update(over)
    return L.ap_sparse_attn_fwd(a["Q"], a["K"], a["V"], a["O"], a["lse"], a["dtype"], a["B"], a["H"],
                                a["Lq"], a["Lk"], a["D"], a["sq"], a["sk"], a["sv"], a["so"],
                                a["row_ptr"], a["col_idx"], a["bitmaps"], a["bm"], a["bn"],
                                a.get("sched"), a["causal"], a["scale"], None)


def test_fwd_rejects_bad_arguments(L):
    assert _fwd(L, Q=None) == ap.AP_ERR_INVALID_ARG
    assert _fwd(L, bitmaps=None) == ap.AP_ERR_INVALID_ARG
    assert _fwd(L, B=0) == ap.AP_ERR_INVALID_ARG
    assert _fwd(L, dtype=7) == ap.AP_ERR_INVALID_ARG
    assert _fwd(L, D=48) == ap.AP_ERR_UNSUPPORTED
    assert _fwd(L, D=256) == ap.AP_ERR_UNSUPPORTED
    assert _fwd(L, bn=32) == ap.AP_ERR_UNSUPPORTED
    assert _fwd(L, bm=32) == ap.AP_ERR_UNSUPPORTED
    assert _fwd(L, bm=128, dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert _fwd(L, causal=1, Lq=128, Lk=64) == ap.AP_ERR_INVALID_ARG          # Lk < Lq with causal
    assert _fwd(L, Q=0x1008) == ap.AP_ERR_INVALID_ARG                          # not 16-byte aligned
    assert _fwd(L, O=0x1000) == ap.AP_ERR_INVALID_ARG                          # O aliases Q
    bad = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 60)
    assert _fwd(L, sk=bad) == ap.AP_ERR_INVALID_ARG                            # row stride not 16-byte multiple
    short = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 32)
    assert _fwd(L, sv=short) == ap.AP_ERR_INVALID_ARG                          # row stride < D
    assert _fwd(L, scale=float("nan")) == ap.AP_ERR_INVALID_ARG


def test_cropped_forward_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)

    def call(**over):
        a = dict(Lq=64, Lk=64, Lql=128, Lkl=128, dtype=ap.AP_BF16, causal=0, sched=None)
        a.update(over)
        return L.ap_sparse_attn_fwd_cropped(fake, fake + 0x100000, fake + 0x200000, fake + 0x300000, None,
                                            a["dtype"], 1, 2, a["Lq"], a["Lk"], 64, s, s, s, s, fake, fake, fake,
                                            64, 64, a["Lql"], a["Lkl"], a["sched"], a["causal"], 0.0, None)

    assert call(Lql=0) == ap.AP_ERR_INVALID_ARG
    assert call(Lql=32) == ap.AP_ERR_INVALID_ARG              # layout smaller than the call
    assert call(Lkl=63) == ap.AP_ERR_INVALID_ARG
    assert call(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    cs = ap._CSchedule(fake, fake, fake, fake)
    # causal with a schedule: the offsets Lk - Lq of call and layout must agree
    assert call(causal=1, Lq=32, Lk=64, sched=ctypes.byref(cs)) == ap.AP_ERR_INVALID_ARG
    assert call(causal=1, Lql=128, Lkl=64) == ap.AP_ERR_INVALID_ARG


def test_schedule_arguments(L):
    fake = 0x1000
    good = ap._CSchedule(fake, fake, fake, fake)
    call = L.ap_build_schedule
    import ctypes as C
    assert call(fake, fake, fake, 2, 64, 64, 64, 64, 8, 0, 0, None, None) == ap.AP_ERR_INVALID_ARG
    assert call(None, fake, fake, 2, 64, 64, 64, 64, 8, 0, 0, C.byref(good), None) == ap.AP_ERR_INVALID_ARG
    assert call(fake, fake, fake, 2, 64, 64, 32, 64, 8, 0, 0, C.byref(good), None) == ap.AP_ERR_UNSUPPORTED
    assert call(fake, fake, fake, 2, 64, 64, 64, 32, 8, 0, 0, C.byref(good), None) == ap.AP_ERR_UNSUPPORTED
    assert call(fake, fake, fake, 2, 64, 64, 64, 64, 8, 0, 66, C.byref(good), None) == ap.AP_ERR_INVALID_ARG
    assert call(fake, fake, fake, 2, 128, 64, 64, 64, 8, 1, 0, C.byref(good), None) == ap.AP_ERR_INVALID_ARG
    hole = ap._CSchedule(fake, None, fake, fake)
    assert call(fake, fake, fake, 2, 64, 64, 64, 64, 8, 0, 0, C.byref(hole), None) == ap.AP_ERR_INVALID_ARG
    # forward: a schedule needs bf16 and complete pointers
    assert _fwd(L, sched=C.pointer(hole)) == ap.AP_ERR_INVALID_ARG
    assert _fwd(L, sched=C.pointer(good), dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    # gathered rows are addressed with a 24-bit multiply: lengths and row strides in bytes below 2^24
    wide = (ctypes.c_int64 * 3)(2 * 64 * (1 << 23), 64 * (1 << 23), 1 << 23)
    assert _fwd(L, sched=C.pointer(good), sk=wide) == ap.AP_ERR_UNSUPPORTED
    assert _fwd(L, sched=C.pointer(good), Lk=1 << 24, D=32) == ap.AP_ERR_UNSUPPORTED


def test_mask_construction_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)
    assert ap.ap_attention_maps_workspace_bytes(4, 16, 4096) == 4 * 16 * 4096 * 4
    assert ap.ap_attention_maps_workspace_bytes(0, 16, 4096) == 0
    ws = ap.ap_attention_maps_workspace_bytes(1, 2, 64)

    def acc(**over):
        a = dict(Q=fake, K=fake + 0x100000, dtype=ap.AP_BF16, B=1, H=2, Lq=64, Lk=64, D=64, sq=s, sk=s,
                 causal=0, scale=0.0, weight=1.0, abar=fake, ws=fake, ws_bytes=ws)
        a.update(over)
        return L.ap_accumulate_attention_maps(a["Q"], a["K"], a["dtype"], a["B"], a["H"], a["Lq"],
                                              a["Lk"], a["D"], a["sq"], a["sk"], a["causal"], a["scale"],
                                              a["weight"], a["abar"], a["ws"], a["ws_bytes"], None)

    assert acc(Q=None) == ap.AP_ERR_INVALID_ARG
    assert acc(abar=None) == ap.AP_ERR_INVALID_ARG
    assert acc(ws=None) == ap.AP_ERR_INVALID_ARG
    assert acc(H=0) == ap.AP_ERR_INVALID_ARG
    assert acc(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert acc(D=48) == ap.AP_ERR_UNSUPPORTED
    assert acc(causal=1, Lq=128, Lk=64) == ap.AP_ERR_INVALID_ARG
    assert acc(abar=0x1004) == ap.AP_ERR_INVALID_ARG
    assert acc(weight=float("inf")) == ap.AP_ERR_INVALID_ARG
    assert acc(ws_bytes=ws - 1) == ap.AP_ERR_CAPACITY
    bad = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 60)
    assert acc(sk=bad) == ap.AP_ERR_INVALID_ARG

    def acc_lse(lse=fake + 0x200000, **over):
        a = dict(Q=fake, ws_bytes=ws, dtype=ap.AP_BF16)
        a.update(over)
        return L.ap_accumulate_attention_maps_lse(a["Q"], fake + 0x100000, lse, a["dtype"], 1, 2, 64, 64, 64, s, s,
                                                  0, 0.0, 1.0, fake, fake, a["ws_bytes"], None)

    assert acc_lse(lse=None) == ap.AP_ERR_INVALID_ARG
    assert acc_lse(lse=fake + 2) == ap.AP_ERR_INVALID_ARG                      # not 4-byte aligned
    assert acc_lse(Q=None) == ap.AP_ERR_INVALID_ARG
    assert acc_lse(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert acc_lse(ws_bytes=ws - 1) == ap.AP_ERR_CAPACITY

    wp = ap.ap_prune_mask_workspace_bytes()
    assert wp == 64 + 32768 * 8 + (1 << 20) * (4 + 8)      # state, histogram, candidate keys and indices

    def prune(**over):
        a = dict(abar=fake, H=2, Lq=64, Lk=64, causal=0, p=0.9, mask=fake, tau=fake, ws=fake, ws_bytes=wp)
        a.update(over)
        return L.ap_prune_mask(a["abar"], a["H"], a["Lq"], a["Lk"], a["causal"], a["p"], a["mask"],
                               a["tau"], a["ws"], a["ws_bytes"], None)

    assert prune(abar=None) == ap.AP_ERR_INVALID_ARG
    assert prune(mask=None, tau=None) == ap.AP_ERR_INVALID_ARG    # nothing to write (mask = NULL alone: threshold only)
    assert prune(Lk=0) == ap.AP_ERR_INVALID_ARG
    assert prune(p=-0.1) == ap.AP_ERR_INVALID_ARG
    assert prune(p=1.5) == ap.AP_ERR_INVALID_ARG
    assert prune(p=float("nan")) == ap.AP_ERR_INVALID_ARG
    assert prune(causal=1, Lq=128, Lk=64) == ap.AP_ERR_INVALID_ARG
    assert prune(abar=0x1004) == ap.AP_ERR_INVALID_ARG
    assert prune(mask=0x1002) == ap.AP_ERR_INVALID_ARG
    assert prune(ws_bytes=wp - 1) == ap.AP_ERR_CAPACITY


def test_split_forward_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)
    assert ap.ap_fwd_split_workspace_bytes(4, 16, 64, 128, 8) == 8 * 4 * 16 * 64 * 129 * 4
    assert ap.ap_fwd_split_workspace_bytes(4, 16, 64, 128, 0) == 0
    ws = ap.ap_fwd_split_workspace_bytes(1, 2, 64, 64, 4)

    def call(**over):
        a = dict(Q=fake, K=fake + 0x100000, V=fake + 0x200000, O=fake + 0x300000, dtype=ap.AP_BF16, bm=64,
                 splits=4, ws=fake, ws_bytes=ws, sq=s)
        a.update(over)
        return L.ap_sparse_attn_fwd_split(a["Q"], a["K"], a["V"], a["O"], None, a["dtype"], 1, 2, 64, 64, 64,
                                          a["sq"], s, s, s, fake, fake, fake, a["bm"], 64, None, 0, 0.0,
                                          a["splits"], a["ws"], a["ws_bytes"], None)

    assert call(splits=0) == ap.AP_ERR_INVALID_ARG
    assert call(Q=None) == ap.AP_ERR_INVALID_ARG
    assert call(ws=None) == ap.AP_ERR_INVALID_ARG
    assert call(ws=0x1008) == ap.AP_ERR_INVALID_ARG
    assert call(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert call(bm=128) == ap.AP_ERR_UNSUPPORTED
    assert call(splits=2000) == ap.AP_ERR_UNSUPPORTED
    assert call(ws_bytes=ws - 1) == ap.AP_ERR_CAPACITY
    bad = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 60)
    assert call(sq=bad) == ap.AP_ERR_INVALID_ARG


def test_static_split_forward_rejects_sizes_beyond_its_array(L):
    """The allocation-free variant checks its fixed capacity on the host before anything else."""
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)

    def call(B, H, Lq, D, splits):
        return L.ap_sparse_attn_fwd_split_static(fake, fake + 0x100000, fake + 0x200000, fake + 0x300000, None,
                                                 ap.AP_BF16, B, H, Lq, 64, D, s, s, s, s, fake, fake, fake,
                                                 64, 64, None, 0, 0.0, splits, None)

    assert call(1, 2, 64, 64, 0) == ap.AP_ERR_INVALID_ARG
    assert call(0, 2, 64, 64, 4) == ap.AP_ERR_INVALID_ARG
    limit = ap.AP_FWD_SPLIT_STATIC_MAX_BYTES
    assert ap.ap_fwd_split_workspace_bytes(4, 16, 64, 128, 16) > limit
    assert call(4, 16, 64, 128, 16) == ap.AP_ERR_CAPACITY
    assert call(65535, 65535, 1 << 30, 128, 1024) == ap.AP_ERR_CAPACITY       # no wrap-around
    text = open(os.path.join(ROOT, "include", "ap.h")).read()
    assert "#define AP_FWD_SPLIT_STATIC_MAX_BYTES ((size_t)32 << 20)" in text and limit == 32 << 20


def test_entmax_forward_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)

    def call(**over):
        a = dict(Q=fake, K=fake + 0x100000, V=fake + 0x200000, O=fake + 0x300000, dtype=ap.AP_BF16, bm=64, D=64,
                 causal=0, Lq=64, Lk=64, sched=None)
        a.update(over)
        return L.ap_sparse_attn_entmax15_fwd(a["Q"], a["K"], a["V"], a["O"], None, a["dtype"], 1, 2, a["Lq"],
                                             a["Lk"], a["D"], s, s, s, s, fake, fake, fake, a["bm"], 64,
                                             a["sched"], a["causal"], 0.0, None)

    assert call(K=None) == ap.AP_ERR_INVALID_ARG
    assert call(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert call(bm=128) == ap.AP_ERR_UNSUPPORTED
    assert call(D=48) == ap.AP_ERR_UNSUPPORTED
    assert call(causal=1, Lq=128, Lk=64) == ap.AP_ERR_INVALID_ARG
    assert call(O=fake) == ap.AP_ERR_INVALID_ARG
    hole = ap._CSchedule(fake, None, fake, fake)
    assert call(sched=ctypes.pointer(hole)) == ap.AP_ERR_INVALID_ARG


def test_backward_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)
    assert ap.ap_bwd_workspace_bytes(4, 16, 4096) == 4 * 16 * 4096 * 4
    assert ap.ap_bwd_workspace_bytes(4, 0, 4096) == 0
    ws = ap.ap_bwd_workspace_bytes(1, 2, 64)

    def bwd(**over):
        a = dict(Q=fake, K=fake + 0x100000, V=fake + 0x200000, O=fake + 0x300000, dO=fake + 0x400000,
                 lse=fake + 0x500000, dQ=fake + 0x600000, dK=fake + 0x700000, dV=fake + 0x800000,
                 dtype=ap.AP_BF16, B=1, H=2, Lq=64, Lk=64, D=64, sq=s, sk=s, sv=s, so=s, row_ptr=fake,
                 col_idx=fake, bitmaps=fake, col_ptr=fake, row_idx=fake, tile_idx=fake, bm=64, bn=64,
                 causal=0, scale=0.0, ws=fake, ws_bytes=ws)
        a.update(over)
        return L.ap_sparse_attn_bwd(a["Q"], a["K"], a["V"], a["O"], a["dO"], a["lse"], a["dQ"], a["dK"],
                                    a["dV"], a["dtype"], a["B"], a["H"], a["Lq"], a["Lk"], a["D"], a["sq"],
                                    a["sk"], a["sv"], a["so"], a["row_ptr"], a["col_idx"], a["bitmaps"],
                                    a["col_ptr"], a["row_idx"], a["tile_idx"], a["bm"], a["bn"],
                                    a["causal"], a["scale"], a["ws"], a["ws_bytes"], None)

    assert bwd(dO=None) == ap.AP_ERR_INVALID_ARG
    assert bwd(lse=None) == ap.AP_ERR_INVALID_ARG
    assert bwd(col_ptr=None) == ap.AP_ERR_INVALID_ARG
    assert bwd(ws=None) == ap.AP_ERR_INVALID_ARG
    assert bwd(B=0) == ap.AP_ERR_INVALID_ARG
    assert bwd(dQ=fake) == ap.AP_ERR_INVALID_ARG                               # dQ aliases Q
    assert bwd(dV=fake + 0x700000) == ap.AP_ERR_INVALID_ARG                    # dV aliases dK
    assert bwd(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert bwd(D=48) == ap.AP_ERR_UNSUPPORTED
    assert bwd(bm=128) == ap.AP_ERR_UNSUPPORTED
    assert bwd(causal=1, Lq=128, Lk=64) == ap.AP_ERR_INVALID_ARG
    assert bwd(dK=fake + 0x700008) == ap.AP_ERR_INVALID_ARG                    # not 16-byte aligned
    assert bwd(ws_bytes=ws - 1) == ap.AP_ERR_CAPACITY
    bad = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 60)
    assert bwd(so=bad) == ap.AP_ERR_INVALID_ARG

    tr = L.ap_build_layout_transpose
    assert tr(None, fake, 2, 64, 64, 64, 64, 8, fake, fake, fake, None) == ap.AP_ERR_INVALID_ARG
    assert tr(fake, fake, 2, 64, 64, 64, 64, 8, fake, None, fake, None) == ap.AP_ERR_INVALID_ARG
    assert tr(fake, fake, 0, 64, 64, 64, 64, 8, fake, fake, fake, None) == ap.AP_ERR_INVALID_ARG
    assert tr(fake, fake, 2, 64, 64, 48, 64, 8, fake, fake, fake, None) == ap.AP_ERR_UNSUPPORTED
    assert tr(fake, fake, 2, 64, 64, 64, 64, -1, fake, fake, fake, None) == ap.AP_ERR_INVALID_ARG
    assert tr(fake, fake + 2, 2, 64, 64, 64, 64, 8, fake, fake, fake, None) == ap.AP_ERR_INVALID_ARG


def test_scheduled_backward_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)
    ws = ap.ap_bwd_workspace_bytes(1, 2, 64)
    good = ap._CSchedule(fake, fake, fake, fake)
    hole = ap._CSchedule(fake, None, fake, fake)
    odd = ap._CSchedule(fake, fake, fake, fake + 4)                            # bitmaps not 8-byte aligned

    def bwd(sched, col_sched, **over):
        a = dict(dtype=ap.AP_BF16, bm=64, causal=0, Lq=64, Lk=64)
        a.update(over)
        ptrs = [fake + i * 0x100000 for i in range(9)]
        return L.ap_sparse_attn_bwd_sched(*ptrs, a["dtype"], 1, 2, a["Lq"], a["Lk"], 64, s, s, s, s, fake, fake,
                                          fake, fake, fake, fake, a["bm"], 64,
                                          ctypes.byref(sched) if sched else None,
                                          ctypes.byref(col_sched) if col_sched else None, a["causal"], 0.0,
                                          fake, ws, None)

    assert bwd(hole, None) == ap.AP_ERR_INVALID_ARG
    assert bwd(None, hole) == ap.AP_ERR_INVALID_ARG
    assert bwd(good, odd) == ap.AP_ERR_INVALID_ARG
    assert bwd(good, good, dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert bwd(good, good, bm=128) == ap.AP_ERR_UNSUPPORTED
    assert bwd(good, good, causal=1, Lq=128) == ap.AP_ERR_INVALID_ARG

    def build(**over):
        a = dict(col_ptr=fake, row_idx=fake, tile_idx=fake, bitmaps=fake, H=2, Lq=64, Lk=64, bm=64, bn=64,
                 cap=8, causal=0, min_rows=0, sched=good)
        a.update(over)
        return L.ap_build_col_schedule(a["col_ptr"], a["row_idx"], a["tile_idx"], a["bitmaps"], a["H"], a["Lq"],
                                       a["Lk"], a["bm"], a["bn"], a["cap"], a["causal"], a["min_rows"],
                                       ctypes.byref(a["sched"]) if a["sched"] else None, None)

    assert build(col_ptr=None) == ap.AP_ERR_INVALID_ARG
    assert build(sched=None) == ap.AP_ERR_INVALID_ARG
    assert build(sched=hole) == ap.AP_ERR_INVALID_ARG
    assert build(sched=odd) == ap.AP_ERR_INVALID_ARG
    assert build(H=0) == ap.AP_ERR_INVALID_ARG
    assert build(cap=-1) == ap.AP_ERR_INVALID_ARG
    assert build(min_rows=66) == ap.AP_ERR_INVALID_ARG
    assert build(min_rows=-1) == ap.AP_ERR_INVALID_ARG
    assert build(causal=1, Lq=128) == ap.AP_ERR_INVALID_ARG
    assert build(bm=128) == ap.AP_ERR_UNSUPPORTED
    assert build(tile_idx=fake + 2) == ap.AP_ERR_INVALID_ARG


def test_entmax_backward_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)
    assert ap.ap_entmax15_bwd_workspace_bytes(4, 16, 4096) == 4 * 16 * 4096 * 4
    assert ap.ap_entmax15_bwd_workspace_bytes(0, 16, 4096) == 0
    ws = ap.ap_entmax15_bwd_workspace_bytes(1, 2, 64)
    good = ap._CSchedule(fake, fake, fake, fake)

    def bwd(sched=good, col_sched=good, **over):
        a = dict(dtype=ap.AP_BF16, D=64, bm=64, tau=fake + 0x900000, ws_bytes=ws, dQ=fake + 0x500000)
        a.update(over)
        ptrs = [fake + i * 0x100000 for i in range(4)]
        return L.ap_sparse_attn_entmax15_bwd(*ptrs, a["tau"], a["dQ"], fake + 0x600000, fake + 0x700000,
                                             a["dtype"], 1, 2, 64, 64, a["D"], s, s, s, s, fake, fake, fake, fake,
                                             fake, fake, a["bm"], 64,
                                             ctypes.byref(sched) if sched else None,
                                             ctypes.byref(col_sched) if col_sched else None, 0, 0.0,
                                             fake, a["ws_bytes"], None)

    assert bwd(sched=None) == ap.AP_ERR_INVALID_ARG                            # both schedules are required
    assert bwd(col_sched=None) == ap.AP_ERR_INVALID_ARG
    assert bwd(tau=None) == ap.AP_ERR_INVALID_ARG
    assert bwd(dQ=fake) == ap.AP_ERR_INVALID_ARG                               # dQ aliases Q
    assert bwd(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert bwd(D=48) == ap.AP_ERR_UNSUPPORTED
    assert bwd(bm=128) == ap.AP_ERR_UNSUPPORTED
    assert bwd(ws_bytes=ws - 1) == ap.AP_ERR_CAPACITY


def test_cropped_layout_arguments(L):
    fake = 0x1000
    ws = ap.ap_layout_workspace_bytes(2, 64, 64, 64, 64)

    def crop(LqS=128, LkS=128, Lq=64, Lk=64, mask=fake, ws_bytes=ws):
        return L.ap_build_layout_cropped(mask, 2, LqS, LkS, Lq, Lk, 64, 64, fake, fake, fake, 8, None, fake,
                                         ws_bytes, None)

    assert crop(Lq=129) == ap.AP_ERR_INVALID_ARG            # the corner must lie inside the stored mask
    assert crop(Lk=200) == ap.AP_ERR_INVALID_ARG
    assert crop(LqS=0) == ap.AP_ERR_INVALID_ARG
    assert crop(Lq=0) == ap.AP_ERR_INVALID_ARG
    assert crop(mask=None) == ap.AP_ERR_INVALID_ARG
    assert crop(ws_bytes=ws - 1) == ap.AP_ERR_CAPACITY


def test_decode_arguments(L):
    fake = 0x1000
    s = (ctypes.c_int64 * 3)(2 * 64 * 64, 64 * 64, 64)

    def dec(**over):
        a = dict(Q=fake, O=fake + 0x300000, dtype=ap.AP_BF16, D=64, bm=64, bn=64, causal=0, Lq=1, Lk=64)
        a.update(over)
        return L.ap_sparse_attn_decode(a["Q"], fake + 0x100000, fake + 0x200000, a["O"], None, a["dtype"], 1, 2,
                                       a["Lq"], a["Lk"], a["D"], s, s, s, s, fake, fake, fake, a["bm"], a["bn"],
                                       a["causal"], 0.0, a.get("splits", 1), a.get("ws", None), a.get("wsb", 0), None)

    assert dec(splits=0) == ap.AP_ERR_INVALID_ARG
    assert dec(splits=4, ws=None) == ap.AP_ERR_INVALID_ARG                     # splits > 1 need a workspace
    assert dec(splits=4, ws=fake, wsb=16) == ap.AP_ERR_CAPACITY
    assert dec(Q=None) == ap.AP_ERR_INVALID_ARG
    assert dec(O=fake) == ap.AP_ERR_INVALID_ARG                                # O aliases Q
    assert dec(dtype=ap.AP_F32) == ap.AP_ERR_UNSUPPORTED
    assert dec(D=48) == ap.AP_ERR_UNSUPPORTED
    assert dec(bn=32) == ap.AP_ERR_UNSUPPORTED
    assert dec(causal=1, Lq=128, Lk=64) == ap.AP_ERR_INVALID_ARG


def test_binding_rejects_caller_supplied_outputs_that_do_not_fit():
    """The C ABI sees only pointers: the binding checks shape, dtype, device and layout of `out`,
    `lse` and `tau` before anything reaches the library (host tensors suffice to show it)."""
    import torch

    B, H, Lq, Lk, D = 2, 2, 64, 64, 32
    q = torch.zeros((B, H, Lq, D), dtype=torch.bfloat16)
    k = torch.zeros((B, H, Lk, D), dtype=torch.bfloat16)
    z32 = torch.zeros(1, dtype=torch.int32)
    lay = ap.Layout(z32, z32, torch.zeros((1, 64, 1), dtype=torch.int64), torch.zeros(1, dtype=torch.int64),
                    H, Lq, Lk, 64, 64)
    bad_outs = [torch.zeros((B, H, Lq, D), dtype=torch.float32),          # dtype
                torch.zeros((B, H, Lq + 1, D), dtype=torch.bfloat16),     # shape
                torch.zeros((B, H, D, Lq), dtype=torch.bfloat16).transpose(2, 3)]   # last stride
    for out in bad_outs:
        for call in (lambda: ap.ap_sparse_attn_fwd(q, k, k, lay, out=out),
                     lambda: ap.ap_sparse_attn_fwd_split(q, k, k, lay, 2, out=out),
                     lambda: ap.ap_sparse_attn_decode(q, k, k, lay, out=out),
                     lambda: ap.ap_sparse_attn_entmax15_fwd(q, k, k, lay, out=out)):
            with pytest.raises(ValueError):
                call()
    bad_lses = [torch.zeros((B, H, Lq), dtype=torch.float64),
                torch.zeros((B, H, Lq + 1), dtype=torch.float32),
                torch.zeros((B, Lq, H), dtype=torch.float32).transpose(1, 2)]
    for lse in bad_lses:
        with pytest.raises(ValueError):
            ap.ap_sparse_attn_fwd(q, k, k, lay, lse=lse)


def test_layout_from_map_arguments(L):
    fake = 0x1000
    ws = ap.ap_layout_workspace_bytes(2, 128, 128, 64, 64)

    def call(**over):
        a = dict(abar=fake, tau=fake + 0x100, H=2, Lq=128, Lk=128, causal=0, bm=64, bn=64, rp=fake, ci=fake,
                 bmp=fake, cap=8, ws=fake, ws_bytes=ws)
        a.update(over)
        return L.ap_build_layout_from_map(a["abar"], a["tau"], a["H"], a["Lq"], a["Lk"], a["causal"], a["bm"],
                                          a["bn"], a["rp"], a["ci"], a["bmp"], a["cap"], None, a["ws"],
                                          a["ws_bytes"], None)

    assert call(abar=None) == ap.AP_ERR_INVALID_ARG
    assert call(tau=None) == ap.AP_ERR_INVALID_ARG
    assert call(H=0) == ap.AP_ERR_INVALID_ARG
    assert call(bn=32) == ap.AP_ERR_UNSUPPORTED
    assert call(bm=48) == ap.AP_ERR_UNSUPPORTED
    assert call(causal=1, Lq=128, Lk=64) == ap.AP_ERR_INVALID_ARG
    assert call(ci=None) == ap.AP_ERR_INVALID_ARG            # col_idx and bitmaps go together
    assert call(cap=-1) == ap.AP_ERR_INVALID_ARG
    assert call(ws_bytes=ws - 1) == ap.AP_ERR_CAPACITY
    assert call(tau=fake + 2) == ap.AP_ERR_INVALID_ARG


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(ap, "_lib", None)
    monkeypatch.setattr(ap, "LIB_PATH", "/nonexistent/libap_mi355x.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        ap.lib()


def test_build_reports_kernel_resources_and_no_spills():
    """The build parses the compiler's per-kernel resource remarks and records them; no kernel of
    the built library may spill vector registers (a reload inside a tile loop waits for the tile
    loads in flight)."""
    from paper_2012_02030_amd import build as b

    sample = "\n".join([
        "x.hip:1:1: remark: Function Name: k1 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:1:1: remark:     VGPRs: 12 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:1:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:9:1: remark: Function Name: k2 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:9:1: remark:     VGPRs Spill: 7 [-Rpass-analysis=kernel-resource-usage]",
        "warning: something else",
    ])
    ks = b.kernel_resources(sample)
    assert [k["name"] for k in ks] == ["k1", "k2"]
    assert ks[0]["VGPRs"] == "12" and ks[0]["VGPRs Spill"] == "0" and ks[1]["VGPRs Spill"] == "7"
    # the figures of the library that is loaded by the tests, if it was built in this tree
    if os.path.exists(b.RESOURCES):
        lines = open(b.RESOURCES).read().splitlines()
        assert len(lines) > 20
        assert all("spilled VGPRs 0" in line for line in lines), [l for l in lines if "spilled VGPRs 0" not in l]
