"""ctypes binding of the C boundary declared in include/pruner.h.

Argument marshalling only.  Device buffers are torch tensors on the GPU (PyTorch supplies memory and
streams, nothing else); descriptors are the dataclasses of the `workloads` package or anything with the
same attribute names.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpruner_hip.so")

NO_COMPUTE_PENALTY = 1
NO_MEMORY_PENALTY = 2
REFERENCE_ROUNDING = 4
FUSED_ARITHMETIC = 8
NSYM = 12
SYMBOL_NAMES = ("S1", "S2", "S3", "S4", "S6", "S8", "S5_in0", "S7_in0", "S5_in1", "S7_in1", "S5_out", "S7_out")
WS_DRAFT, WS_TOPK, WS_VERIFY, WS_PRIOR_FILTER, WS_LSE, WS_PACM = 0, 1, 2, 3, 4, 5


class PrunerError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class CDevice(C.Structure):
    _fields_ = [("T_p", C.c_float), ("T_m", C.c_float), ("m_l0", C.c_int32), ("m_l1", C.c_int32),
                ("pu_l1", C.c_int32), ("n_l1", C.c_int32), ("pu_l2", C.c_int32), ("n_l2", C.c_int32)]


class CDim(C.Structure):
    _fields_ = [("axis", C.c_int32 * 2), ("coef", C.c_int32 * 2)]


class CBuffer(C.Structure):
    _fields_ = [("ndim", C.c_int32), ("dim", CDim * 4)]


class CSubgraph(C.Structure):
    _fields_ = [("n_sp", C.c_int32), ("n_rd", C.c_int32), ("extent", C.c_int32 * 7),
                ("sp_levels", C.c_int32), ("rd_levels", C.c_int32), ("dtype_bytes", C.c_int32),
                ("frag", C.c_int32 * 3), ("n_in", C.c_int32), ("inp", CBuffer * 2), ("out", CBuffer), ("hw", CDevice)]


class CPacm(C.Structure):
    _fields_ = [("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p), ("We", C.c_void_p), ("be", C.c_void_p),
                ("Wq", C.c_void_p), ("Wk", C.c_void_p), ("Wv", C.c_void_p), ("Wo", C.c_void_p), ("Wh", C.c_void_p), ("bh", C.c_void_p),
                ("wo", C.c_void_p), ("bo", C.c_float)]


class CMlp(C.Structure):
    _fields_ = [("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p), ("w3", C.c_void_p),
                ("b3", C.c_float)]


_lib = None


def library_path():
    return _LIB_PATH


def load_library():
    """Load libpruner_hip.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2402_02361_amd.build` "
                              "(or __graft_entry__.build()); there is no CPU fallback")
        lib = C.CDLL(_LIB_PATH)
        P = C.POINTER
        lib.pruner_draft_score.restype = C.c_int
        lib.pruner_draft_score.argtypes = [P(CSubgraph), C.c_int32, P(C.c_int64), C.c_void_p, C.c_int64, C.c_int32,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.pruner_topk.restype = C.c_int
        lib.pruner_topk.argtypes = [C.c_void_p, P(C.c_int64), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
        lib.pruner_topk_static.restype = C.c_int
        lib.pruner_topk_static.argtypes = [C.c_void_p, P(C.c_int64), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.pruner_prior_filter.restype = C.c_int
        lib.pruner_prior_filter.argtypes = [P(CSubgraph), C.c_int32, P(C.c_int64), C.c_void_p, C.c_int64, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        lib.pruner_random_init_workspace_bytes.restype = C.c_size_t
        lib.pruner_random_init_workspace_bytes.argtypes = [P(CSubgraph), C.c_int32]
        lib.pruner_random_init.restype = C.c_int
        lib.pruner_random_init.argtypes = [P(CSubgraph), C.c_int32, P(C.c_int64), C.c_void_p, C.c_int64, C.c_int32, C.c_uint64,
                                           C.c_void_p, C.c_size_t, C.c_void_p]
        lib.pruner_moa_update.restype = C.c_int
        lib.pruner_moa_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p]
        lib.pruner_time_dominant_draft_launch.restype = C.c_int
        lib.pruner_time_dominant_draft_launch.argtypes = [C.c_void_p, C.c_void_p, P(C.c_int64)]
        lib.pruner_pacm_score.restype = C.c_int
        lib.pruner_pacm_score.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, P(CPacm), C.c_void_p, C.c_void_p, C.c_size_t,
                                          C.c_void_p]
        lib.pruner_lse.restype = C.c_int
        lib.pruner_lse.argtypes = [P(CSubgraph), C.c_int32, P(C.c_int64), C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                   C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.pruner_verify_score.restype = C.c_int
        lib.pruner_verify_score.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, P(CMlp), C.c_void_p,
                                            C.c_void_p, C.c_size_t, C.c_void_p]
        lib.pruner_workspace_bytes.restype = C.c_size_t
        lib.pruner_workspace_bytes.argtypes = [C.c_int32, C.c_int64, C.c_int32, C.c_int32]
        lib.pruner_strerror.restype = C.c_char_p
        lib.pruner_strerror.argtypes = [C.c_int]
        _lib = lib
    return _lib


def strerror(code):
    return load_library().pruner_strerror(int(code)).decode()


def workspace_bytes(which, n, n_sg, k):
    return int(load_library().pruner_workspace_bytes(which, n, n_sg, k))


def _c_buffer(b):
    out = CBuffer()
    out.ndim = len(b.dims)
    for d in range(4):
        out.dim[d].axis[:] = [-1, -1]
        out.dim[d].coef[:] = [0, 0]
    for d, terms in enumerate(b.dims):
        for t, (axis, coef) in enumerate(terms):
            out.dim[d].axis[t] = axis
            out.dim[d].coef[t] = coef
    return out


def to_c_subgraphs(subgraphs):
    """Marshal descriptors (workloads.Subgraph or look-alikes) into a C array of pruner_subgraph."""
    arr = (CSubgraph * len(subgraphs))()
    for i, sg in enumerate(subgraphs):
        s = arr[i]
        s.n_sp, s.n_rd = sg.n_sp, sg.n_rd
        for a, e in enumerate(sg.extent):
            s.extent[a] = e
        s.sp_levels, s.rd_levels, s.dtype_bytes = sg.sp_levels, sg.rd_levels, sg.dtype_bytes
        s.frag[:] = list(sg.frag)
        s.n_in = len(sg.inputs)
        for j, b in enumerate(sg.inputs):
            s.inp[j] = _c_buffer(b)
        if len(sg.inputs) < 2:
            s.inp[1] = CBuffer()
        s.out = _c_buffer(sg.out)
        h = sg.hw
        s.hw = CDevice(h.T_p, h.T_m, h.m_l0, h.m_l1, h.pu_l1, h.n_l1, h.pu_l2, h.n_l2)
    return arr


def _seg(seg_off):
    seg = np.ascontiguousarray(seg_off, dtype=np.int64)
    return seg, seg.ctypes.data_as(C.POINTER(C.c_int64))


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _workspace(workspace, need, device):
    import torch
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def draft_score(subgraphs, seg_off, tiles, flags=0, score=None, symbols=False, workspace=None, stream=None):
    """pruner_draft_score.  tiles: uint16 CUDA tensor [slots, pitch].  Returns score (and symbols int64 [12, n])."""
    import torch
    lib = load_library()
    assert tiles.is_cuda and tiles.dtype == torch.uint16 and tiles.dim() == 2 and tiles.is_contiguous()
    seg, seg_p = _seg(seg_off)
    n_sg, n = len(seg) - 1, int(seg[-1])
    arr = subgraphs if isinstance(subgraphs, C.Array) else to_c_subgraphs(subgraphs)
    if score is None:
        score = torch.empty(n, dtype=torch.float32, device=tiles.device)
    sym = torch.empty((NSYM, n), dtype=torch.int64, device=tiles.device) if symbols is True else (symbols or None)
    need = workspace_bytes(WS_DRAFT, n, n_sg, 0)
    ws = _workspace(workspace, need, tiles.device)
    rc = lib.pruner_draft_score(arr, n_sg, seg_p, _ptr(tiles), tiles.shape[1], flags, _ptr(score), _ptr(sym),
                                _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_draft_score")
    return (score, sym) if sym is not None else score


def topk(score, seg_off, k, idx_out=None, val_out=None, want_values=True, workspace=None, stream=None):
    """pruner_topk.  score: float32 CUDA tensor [n].  Returns (idx int32 [n_sg, k], val float32 [n_sg, k] or None)."""
    import torch
    lib = load_library()
    assert score.is_cuda and score.dtype == torch.float32 and score.is_contiguous()
    seg, seg_p = _seg(seg_off)
    n_sg, n = len(seg) - 1, int(seg[-1])
    if idx_out is None:
        idx_out = torch.empty((max(n_sg, 0), max(k, 0)), dtype=torch.int32, device=score.device)
    if val_out is None and want_values:
        val_out = torch.empty((max(n_sg, 0), max(k, 0)), dtype=torch.float32, device=score.device)
    need = workspace_bytes(WS_TOPK, n, n_sg, k)
    ws = _workspace(workspace, need, score.device)
    rc = lib.pruner_topk(_ptr(score), seg_p, n_sg, k, _ptr(idx_out), _ptr(val_out), _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_topk")
    return idx_out, val_out


def topk_static(score, seg_off, k, idx_out, val_out=None, stream=None):
    """pruner_topk_static: pruner_topk with the scratch inside the library; the caller passes every buffer (nothing is allocated
    here either).  Returns (idx_out, val_out)."""
    import torch
    lib = load_library()
    assert score.is_cuda and score.dtype == torch.float32 and score.is_contiguous()
    seg, seg_p = _seg(seg_off)
    rc = lib.pruner_topk_static(_ptr(score), seg_p, len(seg) - 1, k, _ptr(idx_out), _ptr(val_out), _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_topk_static")
    return idx_out, val_out


def prior_filter(subgraphs, seg_off, tiles, k, flags=0, score=None, idx_out=None, val_out=None, want_values=True, workspace=None,
                 stream=None, scored_event=None):
    """pruner_prior_filter.  Returns (score float32 [n], idx int32 [n_sg, k], val float32 [n_sg, k] or None).
    scored_event: a torch.cuda.Event that has been recorded once already (its handle must exist), or None."""
    import torch
    lib = load_library()
    assert tiles.is_cuda and tiles.dtype == torch.uint16 and tiles.dim() == 2 and tiles.is_contiguous()
    seg, seg_p = _seg(seg_off)
    n_sg, n = len(seg) - 1, int(seg[-1])
    arr = subgraphs if isinstance(subgraphs, C.Array) else to_c_subgraphs(subgraphs)
    if score is None:
        score = torch.empty(n, dtype=torch.float32, device=tiles.device)
    if idx_out is None:
        idx_out = torch.empty((max(n_sg, 0), max(k, 0)), dtype=torch.int32, device=tiles.device)
    if val_out is None and want_values:
        val_out = torch.empty((max(n_sg, 0), max(k, 0)), dtype=torch.float32, device=tiles.device)
    need = workspace_bytes(WS_PRIOR_FILTER, n, n_sg, k)
    ws = _workspace(workspace, need, tiles.device)
    ev = C.c_void_p(scored_event.cuda_event) if scored_event is not None else None
    rc = lib.pruner_prior_filter(arr, n_sg, seg_p, _ptr(tiles), tiles.shape[1], flags, k, _ptr(score), _ptr(idx_out), _ptr(val_out),
                                 _ptr(ws), ws.numel(), _stream(stream), ev)
    if rc:
        raise PrunerError(rc, "pruner_prior_filter")
    return score, idx_out, val_out


def lse(subgraphs, seg_off, tiles, k, n_steps, seed, mutate_q16, flags=0, score=None, workspace=None, stream=None):
    """pruner_lse.  tiles (uint16 CUDA [rows, pitch]) is updated in place.  Returns (score float32 [n],
    spec_tiles uint16 [rows, n_sg * k], spec_score float32 [n_sg, k], spec_count int32 [n_sg])."""
    import torch
    lib = load_library()
    assert tiles.is_cuda and tiles.dtype == torch.uint16 and tiles.dim() == 2 and tiles.is_contiguous()
    seg, seg_p = _seg(seg_off)
    n_sg, n = len(seg) - 1, int(seg[-1])
    arr = subgraphs if isinstance(subgraphs, C.Array) else to_c_subgraphs(subgraphs)
    if score is None:
        score = torch.empty(n, dtype=torch.float32, device=tiles.device)
    rows = tiles.shape[0]
    spec_tiles = torch.empty((rows, max(n_sg * k, 0)), dtype=torch.uint16, device=tiles.device)
    spec_score = torch.empty((max(n_sg, 0), max(k, 0)), dtype=torch.float32, device=tiles.device)
    spec_count = torch.empty(max(n_sg, 0), dtype=torch.int32, device=tiles.device)
    need = workspace_bytes(WS_LSE, n, n_sg, k)
    ws = _workspace(workspace, need, tiles.device)
    rc = lib.pruner_lse(arr, n_sg, seg_p, _ptr(tiles), tiles.shape[1], rows, flags, k, n_steps, seed & 0xFFFFFFFFFFFFFFFF, mutate_q16,
                        _ptr(score), _ptr(spec_tiles), _ptr(spec_score), _ptr(spec_count), _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_lse")
    return score, spec_tiles, spec_score, spec_count


def random_init(subgraphs, seg_off, rows, seed, tiles=None, workspace=None, stream=None, device="cuda"):
    """pruner_random_init.  Returns tiles (uint16 CUDA [rows, pitch]; a given tensor is filled in place)."""
    import torch
    lib = load_library()
    seg, seg_p = _seg(seg_off)
    n_sg, n = len(seg) - 1, int(seg[-1])
    arr = subgraphs if isinstance(subgraphs, C.Array) else to_c_subgraphs(subgraphs)
    if tiles is None:
        tiles = torch.empty((rows, n), dtype=torch.uint16, device=device)
    assert tiles.is_cuda and tiles.dtype == torch.uint16 and tiles.dim() == 2 and tiles.is_contiguous() and tiles.shape[0] == rows
    need = int(lib.pruner_random_init_workspace_bytes(arr, n_sg))
    ws = _workspace(workspace, max(need, 256), tiles.device)
    rc = lib.pruner_random_init(arr, n_sg, seg_p, _ptr(tiles), tiles.shape[1], rows, seed & 0xFFFFFFFFFFFFFFFF, _ptr(ws), ws.numel(),
                                _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_random_init")
    return tiles


def pacm_score(feat, n_stmt, flow, n_blk, weights, y=None, workspace=None, stream=None):
    """pruner_pacm_score.  feat float32 CUDA [n_d, 8, 164], n_stmt int32 CUDA [n_d]; flow float32 CUDA [n_d, 8, 23], n_blk
    int32 CUDA [n_d]; weights: dict of CUDA tensors W1 b1 W2 b2 We be Wq Wk Wv Wo Wh bh wo (matrices uint16 bf16 bits or
    torch.bfloat16, biases float32) and float bo."""
    import torch
    lib = load_library()
    n_d = feat.shape[0]
    assert feat.is_cuda and feat.dtype == torch.float32 and feat.is_contiguous() and feat.shape[1:] == (8, 164)
    assert flow.is_cuda and flow.dtype == torch.float32 and flow.is_contiguous() and flow.shape == (n_d, 8, 23)
    assert n_stmt.is_cuda and n_stmt.dtype == torch.int32 and n_stmt.is_contiguous() and n_stmt.numel() == n_d
    assert n_blk.is_cuda and n_blk.dtype == torch.int32 and n_blk.is_contiguous() and n_blk.numel() == n_d
    if y is None:
        y = torch.empty(n_d, dtype=torch.float32, device=feat.device)
    names = ("W1", "b1", "W2", "b2", "We", "be", "Wq", "Wk", "Wv", "Wo", "Wh", "bh", "wo")
    m = CPacm(*[weights[k].data_ptr() for k in names], float(weights["bo"]))
    need = workspace_bytes(WS_PACM, n_d, 0, 0)
    ws = _workspace(workspace, need, feat.device)
    rc = lib.pruner_pacm_score(_ptr(feat), _ptr(n_stmt), _ptr(flow), _ptr(n_blk), n_d, C.byref(m), _ptr(y), _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_pacm_score")
    return y


def moa_update(phi_s, phi_t, m, bf16=None, stream=None):
    """pruner_moa_update.  phi_s (float32 CUDA, updated in place), phi_t (float32 CUDA, same size); bf16: a uint16 CUDA
    tensor of the same size that receives the new phi_s as bfloat16 bits, or None."""
    import torch
    lib = load_library()
    assert phi_s.is_cuda and phi_s.dtype == torch.float32 and phi_s.is_contiguous()
    assert phi_t.is_cuda and phi_t.dtype == torch.float32 and phi_t.is_contiguous() and phi_t.numel() == phi_s.numel()
    if bf16 is not None:
        assert bf16.is_cuda and bf16.dtype == torch.uint16 and bf16.is_contiguous() and bf16.numel() == phi_s.numel()
    rc = lib.pruner_moa_update(_ptr(phi_s), _ptr(phi_t), phi_s.numel(), float(m), _ptr(bf16) if bf16 is not None else None, _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_moa_update")
    return phi_s


def time_dominant_draft_launch(start_event=None, stop_event=None, bytes_out=None):
    """pruner_time_dominant_draft_launch.  Events: torch.cuda.Event objects that have been recorded once (so that their
    handles exist), or None for both to switch the hook off; bytes_out: a ctypes.c_int64 that receives the launch's
    algorithmic bytes at every scoring call, or None."""
    lib = load_library()
    a = C.c_void_p(start_event.cuda_event) if start_event is not None else None
    b = C.c_void_p(stop_event.cuda_event) if stop_event is not None else None
    rc = lib.pruner_time_dominant_draft_launch(a, b, C.byref(bytes_out) if bytes_out is not None else None)
    if rc:
        raise PrunerError(rc, "pruner_time_dominant_draft_launch")


def verify_score(feat, n_stmt, weights, vscore=None, workspace=None, stream=None):
    """pruner_verify_score.  feat float32 CUDA [n_d, 8, 164]; n_stmt int32 CUDA [n_d];
    weights: dict of CUDA tensors W1/W2/w3 (uint16 bf16 bits or torch.bfloat16), b1/b2 (float32), and float b3."""
    import torch
    lib = load_library()
    assert feat.is_cuda and feat.dtype == torch.float32 and feat.is_contiguous() and feat.shape[1:] == (8, 164)
    assert n_stmt.is_cuda and n_stmt.dtype == torch.int32 and n_stmt.is_contiguous()
    n_d = feat.shape[0]
    if vscore is None:
        vscore = torch.empty(n_d, dtype=torch.float32, device=feat.device)
    m = CMlp(weights["W1"].data_ptr(), weights["b1"].data_ptr(), weights["W2"].data_ptr(), weights["b2"].data_ptr(),
             weights["w3"].data_ptr(), float(weights["b3"]))
    need = workspace_bytes(WS_VERIFY, n_d, 0, 0)
    ws = _workspace(workspace, need, feat.device)
    rc = lib.pruner_verify_score(_ptr(feat), _ptr(n_stmt), n_d, C.byref(m), _ptr(vscore), _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise PrunerError(rc, "pruner_verify_score")
    return vscore
