"""The C boundary without a GPU: the library loads, exports what include/pruner.h declares, and refuses bad
arguments before anything is launched (every call below returns from host-side validation)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2402_02361_amd as P
import workloads as w

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, EINVAL, EWORKSPACE, ERANGE = 0, -1, -2, -3
FAKE = C.c_void_p(0x1000)          # aligned, never dereferenced on these paths


@pytest.fixture(scope="module")
def lib():
    return P.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "pruner.h")).read()
    names = set(re.findall(r"\b(pruner_[a-z_]+)\s*\(", header))
    assert {"pruner_draft_score", "pruner_topk", "pruner_prior_filter", "pruner_lse", "pruner_random_init",
            "pruner_random_init_workspace_bytes", "pruner_moa_update", "pruner_pacm_score", "pruner_time_dominant_draft_launch", "pruner_verify_score", "pruner_workspace_bytes", "pruner_strerror"} <= names
    for name in names:
        assert hasattr(lib, name), name


def test_struct_sizes_match_the_header():
    # pruner_device 8 x 4 bytes; pruner_dim 16; pruner_buffer 4 + 4*16; pruner_subgraph as laid out in the header
    assert C.sizeof(P.binding.CDevice) == 32 and C.sizeof(P.binding.CDim) == 16 and C.sizeof(P.binding.CBuffer) == 68
    assert C.sizeof(P.CSubgraph) == 4 * (2 + 7 + 2 + 1 + 3 + 1) + 3 * 68 + 32


def test_error_strings(lib):
    assert P.strerror(0) == "ok"
    assert "workspace" in P.strerror(EWORKSPACE) and "invalid" in P.strerror(EINVAL)
    assert P.strerror(-99) == "unknown error code"


def test_workspace_sizes_grow_with_the_problem():
    assert P.workspace_bytes(P.WS_DRAFT, 1000, 1, 0) >= 256
    assert P.workspace_bytes(P.WS_TOPK, 1 << 24, 2, 4096) > P.workspace_bytes(P.WS_TOPK, 1 << 12, 2, 64)
    assert P.workspace_bytes(P.WS_VERIFY, 10240, 0, 0) == 256               # the verify stage keeps its row numbering on chip
    assert P.workspace_bytes(99, 1, 1, 1) == 0


def _draft(lib, sgs, seg, tiles=FAKE, pitch=None, flags=0, score=FAKE, ws=FAKE, ws_bytes=1 << 20):
    arr = P.to_c_subgraphs(sgs)
    seg = np.asarray(seg, dtype=np.int64)
    pitch = int(seg[-1]) if pitch is None else pitch
    return lib.pruner_draft_score(arr, len(sgs), seg.ctypes.data_as(C.POINTER(C.c_int64)), tiles, pitch, flags, score, None,
                                  ws, ws_bytes, None)


def test_draft_score_rejects_bad_arguments(lib):
    g = w.gemm(512, 512, 512)
    assert _draft(lib, [g], [0, 0]) == OK                                    # empty population: nothing to do
    assert _draft(lib, [g], [0, 8], tiles=None) == EINVAL
    assert _draft(lib, [g], [0, 8], score=None) == EINVAL
    assert _draft(lib, [g], [0, 8], tiles=C.c_void_p(0x1001)) == EINVAL      # misaligned
    assert _draft(lib, [g], [0, 8], pitch=4) == EINVAL                       # pitch below n
    assert _draft(lib, [g], [1, 8]) == EINVAL                                # first offset not 0
    assert _draft(lib, [g, g], [0, 8, 4]) == EINVAL                          # decreasing offsets
    assert _draft(lib, [g], [0, 8], flags=16) == EINVAL                      # unknown switch
    assert _draft(lib, [g], [0, 8], flags=4 | 8) == EINVAL                   # both arithmetic switches
    assert _draft(lib, [g], [0, 8], ws=None) == EWORKSPACE
    assert _draft(lib, [g], [0, 8], ws_bytes=16) == EWORKSPACE
    assert _draft(lib, [g], [0, 8], ws=C.c_void_p(0x1010)) == EWORKSPACE     # workspace not 256-byte aligned
    bad = w.Subgraph(**{**g.__dict__, "rd_levels": 4})
    assert _draft(lib, [bad], [0, 8]) == EINVAL
    bad = w.Subgraph(**{**g.__dict__, "extent": (70000, 512, 512)})         # factor would not fit uint16
    assert _draft(lib, [bad], [0, 8]) == EINVAL
    bad = w.gemm(512, 512, 512, hw=w.Device(**{**g.hw.__dict__, "pu_l2": 0}))
    assert _draft(lib, [bad], [0, 8]) == EINVAL
    # symbols that could leave the 32-bit range of the kernel: refused, not computed wrongly
    huge = w.conv2d(64, 512, 224, 224, 512, 3, 3)
    assert _draft(lib, [huge], [0, 8]) == ERANGE


def _topk(lib, seg, k, score=FAKE, idx=FAKE, ws=FAKE, ws_bytes=1 << 30):
    seg = np.asarray(seg, dtype=np.int64)
    return lib.pruner_topk(score, seg.ctypes.data_as(C.POINTER(C.c_int64)), len(seg) - 1, k, idx, None, ws, ws_bytes, None)


def test_topk_static_rejects_bad_arguments(lib):
    def call(seg, k, score=FAKE, idx=FAKE):
        seg = np.asarray(seg, np.int64)
        return lib.pruner_topk_static(score, seg.ctypes.data_as(C.POINTER(C.c_int64)), len(seg) - 1, k, idx, None, None)
    assert call([0, 100], 0) == EINVAL and call([0, 100], 101) == EINVAL and call([0, 10000], 4097) == EINVAL
    assert call([0, 100], 10, score=None) == EINVAL and call([0, 100], 10, idx=None) == EINVAL
    assert call([0, 1 << 31], 10) == EINVAL
    assert call(np.arange(18) * 100, 10) == EINVAL            # 17 segments: above PRUNER_STATIC_MAX_SEGMENTS
    assert call([5, 100], 10) == EINVAL


def test_topk_rejects_bad_arguments(lib):
    assert _topk(lib, [0, 100], 0) == EINVAL
    assert _topk(lib, [0, 100], 101) == EINVAL            # k larger than the segment
    assert _topk(lib, [0, 100, 150], 64) == EINVAL        # ... than any segment
    assert _topk(lib, [0, 10000], 4097) == EINVAL         # above PRUNER_MAX_K
    assert _topk(lib, [0, 100], 10, score=None) == EINVAL
    assert _topk(lib, [0, 100], 10, idx=None) == EINVAL
    assert _topk(lib, [0, 100], 10, ws=None) == EWORKSPACE
    assert _topk(lib, [0, 100], 10, ws_bytes=8) == EWORKSPACE
    assert _topk(lib, [0, 1 << 31], 10) == EINVAL         # indices are int32


def test_prior_filter_rejects_what_its_two_stages_reject(lib):
    g = w.gemm(512, 512, 512)
    arr = P.to_c_subgraphs([g])
    lib.pruner_prior_filter.restype = C.c_int

    def call(seg=(0, 4096), k=64, sgs=arr, tiles=FAKE, score=FAKE, idx=FAKE, ws=FAKE, wsb=1 << 30, flags=0):
        seg = np.asarray(seg, dtype=np.int64)
        return lib.pruner_prior_filter(sgs, 1, seg.ctypes.data_as(C.POINTER(C.c_int64)), tiles, C.c_int64(int(seg[-1])), flags, k, score, idx,
                                       None, ws, C.c_size_t(wsb), None, None)

    assert call(tiles=None) == EINVAL
    assert call(score=None) == EINVAL
    assert call(idx=None) == EINVAL
    assert call(flags=16) == EINVAL and call(flags=12) == EINVAL
    assert call(k=0) == EINVAL
    assert call(k=4097) == EINVAL
    assert call(seg=(0, 32), k=64) == EINVAL                  # fewer candidates than k
    assert call(ws=None) == EWORKSPACE
    assert call(wsb=64) == EWORKSPACE
    assert call(wsb=P.workspace_bytes(P.WS_DRAFT, 4096, 1, 0)) == EWORKSPACE   # room for the draft tables only
    bad = P.to_c_subgraphs([w.conv2d(64, 512, 224, 224, 512, 3, 3)])
    assert call(sgs=bad) == ERANGE
    assert P.workspace_bytes(P.WS_PRIOR_FILTER, 1 << 20, 2, 64) >= (P.workspace_bytes(P.WS_DRAFT, 1 << 20, 2, 0) +
                                                                     P.workspace_bytes(P.WS_TOPK, 1 << 20, 2, 64))


def test_lse_rejects_bad_arguments(lib):
    g = w.gemm(512, 512, 512)
    arr = P.to_c_subgraphs([g])
    lib.pruner_lse.restype = C.c_int

    def call(seg=(0, 4096), k=64, steps=2, q16=40000, rows=10, tiles=FAKE, score=FAKE, spec=FAKE, ws=FAKE, wsb=1 << 30, flags=0, sgs=arr):
        seg = np.asarray(seg, dtype=np.int64)
        return lib.pruner_lse(sgs, 1, seg.ctypes.data_as(C.POINTER(C.c_int64)), tiles, C.c_int64(int(seg[-1])), rows, flags, k, steps,
                              C.c_uint64(1), q16, score, spec, FAKE, FAKE, ws, C.c_size_t(wsb), None)

    assert call(steps=0) == EINVAL
    assert call(q16=65537) == EINVAL
    assert call(k=0) == EINVAL and call(k=4097) == EINVAL
    assert call(rows=9) == EINVAL                       # the GEMM owns 10 slots
    assert call(rows=26) == EINVAL
    assert call(seg=(0, 32)) == EINVAL                  # fewer candidates than k
    assert call(tiles=None) == EINVAL and call(score=None) == EINVAL and call(spec=None) == EINVAL
    assert call(flags=16) == EINVAL and call(flags=12) == EINVAL
    assert call(ws=None) == EWORKSPACE and call(wsb=4096) == EWORKSPACE
    assert call(sgs=P.to_c_subgraphs([w.conv2d(64, 512, 224, 224, 512, 3, 3)]), rows=22) == ERANGE
    assert P.workspace_bytes(P.WS_LSE, 1 << 20, 2, 64) > P.workspace_bytes(P.WS_PRIOR_FILTER, 1 << 20, 2, 64)


def test_random_init_rejects_bad_arguments(lib):
    g = w.gemm(512, 512, 512)
    arr = P.to_c_subgraphs([g])
    need = lib.pruner_random_init_workspace_bytes(arr, 1)
    # three axes of 512: two tables (4 levels: 220 rows, 2 levels: 10 rows) of 8-byte rows, plus the descriptor tables
    assert 230 * 8 <= need < 16384

    def call(seg=(0, 4096), rows=10, tiles=FAKE, pitch=None, ws=FAKE, wsb=1 << 20, sgs=arr, n_sg=1):
        seg = np.asarray(seg, dtype=np.int64)
        return lib.pruner_random_init(sgs, n_sg, seg.ctypes.data_as(C.POINTER(C.c_int64)), tiles, C.c_int64(int(seg[-1]) if pitch is None else pitch),
                                      rows, C.c_uint64(1), ws, C.c_size_t(wsb), None)

    assert call(seg=(0, 0)) == OK                          # empty population: nothing to do
    assert call(sgs=None) == EINVAL
    assert call(seg=(1, 8)) == EINVAL
    assert call(seg=(0, 8, 4), sgs=P.to_c_subgraphs([g, g]), n_sg=2, pitch=8) == EINVAL        # decreasing offsets
    assert call(rows=9) == EINVAL and call(rows=26) == EINVAL
    assert call(tiles=None) == EINVAL
    assert call(tiles=C.c_void_p(0x1001)) == EINVAL
    assert call(pitch=100) == EINVAL
    assert call(ws=None) == EWORKSPACE and call(wsb=need - 1) == EWORKSPACE
    assert call(ws=C.c_void_p(0x1010)) == EWORKSPACE
    bad = P.to_c_subgraphs([w.gemm(64, 72, 64, dtype_bytes=2, rd_levels=3, frag=(16, 16, 16))])   # 72 is no multiple of 16
    assert call(sgs=bad, rows=11) == EINVAL and lib.pruner_random_init_workspace_bytes(bad, 1) == 0
    bad = P.to_c_subgraphs([w.Subgraph(**{**g.__dict__, "extent": (70000, 512, 512)})])
    assert call(sgs=bad) == EINVAL
    # equal axis spaces share a table: twenty subgraphs of one shape need little more than one
    many = P.to_c_subgraphs([g] * 20)
    assert lib.pruner_random_init_workspace_bytes(many, 20) < need + 20 * 512


def test_moa_update_rejects_bad_arguments(lib):
    call = lambda s=FAKE, t=FAKE, n=16, m=0.99, bf=None: lib.pruner_moa_update(s, t, C.c_int64(n), C.c_float(m), bf, None)
    assert call(n=0) == OK
    assert call(n=-1) == EINVAL
    assert call(s=None) == EINVAL and call(t=None) == EINVAL
    assert call(s=C.c_void_p(0x1002)) == EINVAL and call(bf=C.c_void_p(0x1001)) == EINVAL
    assert call(m=1.5) == EINVAL and call(m=-0.1) == EINVAL and call(m=float("nan")) == EINVAL


def test_timing_hook_wants_both_events_or_none(lib):
    lib.pruner_time_dominant_draft_launch.restype = C.c_int
    assert lib.pruner_time_dominant_draft_launch(FAKE, None, None) == EINVAL
    assert lib.pruner_time_dominant_draft_launch(None, FAKE, None) == EINVAL
    assert lib.pruner_time_dominant_draft_launch(None, None, None) == OK


def test_pacm_rejects_bad_arguments(lib):
    full = P.CPacm(*([0x1000] * 13), 0.0)
    call = lambda feat=FAKE, n_stmt=FAKE, flow=FAKE, n_blk=FAKE, n_d=16, mm=full, y=FAKE, ws=FAKE, wsb=1 << 30: lib.pruner_pacm_score(
        feat, n_stmt, flow, n_blk, C.c_int64(n_d), C.byref(mm), y, ws, C.c_size_t(wsb), None)
    assert call(n_d=0) == OK
    assert call(feat=None) == EINVAL and call(flow=None) == EINVAL and call(n_blk=None) == EINVAL and call(y=None) == EINVAL
    assert call(n_d=-1) == EINVAL
    assert call(feat=C.c_void_p(0x1004)) == EINVAL          # feature rows are read 16 bytes at a time
    missing = P.CPacm(*([0x1000] * 6 + [0] + [0x1000] * 6), 0.0)
    assert call(mm=missing) == EINVAL
    assert call(ws=None) == EWORKSPACE and call(wsb=64) == EWORKSPACE
    assert P.workspace_bytes(P.WS_PACM, 1000, 0, 0) >= 1000 * (256 + 64) * 4


def test_verify_rejects_bad_arguments(lib):
    m = P.CMlp(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0.0)
    call = lambda feat=FAKE, n=FAKE, n_d=16, mm=m, out=FAKE, ws=FAKE, wsb=1 << 30: lib.pruner_verify_score(
        feat, n, n_d, C.byref(mm), out, ws, wsb, None)
    assert call(n_d=0) == OK
    assert call(feat=None) == EINVAL and call(out=None) == EINVAL and call(n_d=-1) == EINVAL
    assert call(feat=C.c_void_p(0x1004)) == EINVAL        # feature rows are read 16 bytes at a time
    assert call(mm=P.CMlp(0x1000, 0x1000, 0, 0x1000, 0x1000, 0.0)) == EINVAL
    assert call(ws=None) == EWORKSPACE and call(wsb=64) == EWORKSPACE


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    import paper_2402_02361_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        b.load_library()
