"""Python face of the CPU oracle (oracle/pruner_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package; the HIP library never does, and nothing here imports the HIP package.
The functions marshal numpy arrays into the C oracle and back; all arithmetic
is in the C file, which cites the passages of the paper it follows.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pruner_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

NSYM = 12
SYMBOL_NAMES = ("S1", "S2", "S3", "S4", "S6", "S8", "S5_in0", "S7_in0", "S5_in1", "S7_in1", "S5_out", "S7_out")
TERM_NAMES = ("P0m", "P0c", "P1m", "P1c", "alpha", "P2c", "Ptc", "Up", "Lc",
              "P2m_in0", "Um_in0", "Lm_in0", "P2m_in1", "Um_in1", "Lm_in1", "P2m_out", "Um_out", "Lm_out", "Ltotal")
NO_COMPUTE_PENALTY = 1
NO_MEMORY_PENALTY = 2


def build(force=False):
    """Compile the C oracle with gcc (no contraction of a*b+c into fused multiply-adds)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Device(C.Structure):
    _fields_ = [("T_p", C.c_float), ("T_m", C.c_float), ("m_l0", C.c_int32), ("m_l1", C.c_int32),
                ("pu_l1", C.c_int32), ("n_l1", C.c_int32), ("pu_l2", C.c_int32), ("n_l2", C.c_int32)]


class _Dim(C.Structure):
    _fields_ = [("axis", C.c_int32 * 2), ("coef", C.c_int32 * 2)]


class _Buffer(C.Structure):
    _fields_ = [("ndim", C.c_int32), ("dim", _Dim * 4)]


class _Subgraph(C.Structure):
    _fields_ = [("n_sp", C.c_int32), ("n_rd", C.c_int32), ("extent", C.c_int32 * 7),
                ("sp_levels", C.c_int32), ("rd_levels", C.c_int32), ("dtype_bytes", C.c_int32),
                ("frag", C.c_int32 * 3), ("n_in", C.c_int32), ("inp", _Buffer * 2), ("out", _Buffer), ("hw", _Device)]


def _buffer(b):
    out = _Buffer()
    out.ndim = len(b.dims)
    for d, terms in enumerate(b.dims):
        out.dim[d].axis[:] = [-1, -1]
        out.dim[d].coef[:] = [0, 0]
        for t, (axis, coef) in enumerate(terms):
            out.dim[d].axis[t] = axis
            out.dim[d].coef[t] = coef
    return out


def _subgraph(sg):
    s = _Subgraph()
    s.n_sp, s.n_rd = sg.n_sp, sg.n_rd
    for a, e in enumerate(sg.extent):
        s.extent[a] = e
    s.sp_levels, s.rd_levels, s.dtype_bytes = sg.sp_levels, sg.rd_levels, sg.dtype_bytes
    s.frag[:] = list(sg.frag)
    s.n_in = len(sg.inputs)
    for i, b in enumerate(sg.inputs):
        s.inp[i] = _buffer(b)
    s.out = _buffer(sg.out)
    h = sg.hw
    s.hw = _Device(h.T_p, h.T_m, h.m_l0, h.m_l1, h.pu_l1, h.n_l1, h.pu_l2, h.n_l2)
    return s


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        P = C.POINTER
        lib.orc_analyze_candidate.restype = C.c_int
        lib.orc_analyze_candidate.argtypes = [P(_Subgraph), C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_draft_score.restype = C.c_int
        lib.orc_draft_score.argtypes = [P(_Subgraph), C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_topk.restype = C.c_int
        lib.orc_topk.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.orc_bf16_round.restype = C.c_float
        lib.orc_bf16_round.argtypes = [C.c_float]
        lib.orc_verify.restype = C.c_int
        lib.orc_verify.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
                                   C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_splitmix64_draw.restype = C.c_uint64
        lib.orc_splitmix64_draw.argtypes = [C.c_uint64, C.c_uint64]
        lib.orc_lse.restype = C.c_int
        lib.orc_lse.argtypes = [P(_Subgraph), C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_axis_space.restype = C.c_uint64
        lib.orc_axis_space.argtypes = [P(_Subgraph), C.c_int]
        lib.orc_random_init.restype = C.c_int
        lib.orc_random_init.argtypes = [P(_Subgraph), C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_uint64]
        lib.orc_pacm.restype = C.c_int
        lib.orc_pacm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, P(_PacmWeights), C.c_void_p, C.c_void_p]
        lib.orc_moa_update.restype = C.c_int
        lib.orc_moa_update.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p]
        _lib = lib
    return _lib


class _PacmWeights(C.Structure):
    _fields_ = [("W1", C.c_void_p), ("W2", C.c_void_p), ("b1", C.c_void_p), ("b2", C.c_void_p), ("We", C.c_void_p), ("be", C.c_void_p),
                ("Wq", C.c_void_p), ("Wk", C.c_void_p), ("Wv", C.c_void_p), ("Wo", C.c_void_p), ("Wh", C.c_void_p), ("bh", C.c_void_p),
                ("wo", C.c_void_p), ("bo", C.c_float)]


class OracleError(RuntimeError):
    pass


_ERR = {-1: "bad argument", -2: "tile factors do not multiply to the axis extent", -3: "NaN score", -4: "out of memory"}


def _check(rc):
    if rc:
        raise OracleError(_ERR.get(rc, f"error {rc}"))


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def analyze_candidate(sg, factors, flags=0):
    """Symbols and every intermediate term of one candidate.

    factors: the candidate's tile factors, one per slot.  Returns
    (symbols dict of int, terms64 dict of float, terms32 dict of np.float32).
    """
    f = np.ascontiguousarray(factors, dtype=np.uint16)
    sym = np.zeros(NSYM, dtype=np.int64)
    t64 = np.zeros(len(TERM_NAMES), dtype=np.float64)
    t32 = np.zeros(len(TERM_NAMES), dtype=np.float32)
    s = _subgraph(sg)
    _check(_L().orc_analyze_candidate(C.byref(s), _ptr(f), 1, flags, _ptr(sym), _ptr(t64), _ptr(t32)))
    return (dict(zip(SYMBOL_NAMES, (int(v) for v in sym))), dict(zip(TERM_NAMES, (float(v) for v in t64))),
            dict(zip(TERM_NAMES, t32)))


def draft_score(subgraphs, seg_off, tiles, flags=0, want_symbols=False):
    """Draft fitness F = -L_total of every candidate.

    tiles uint16 [slots, n].  Returns (score32 float32 [n], score64 float64 [n], symbols int64 [12, n] or None).
    """
    tiles = np.ascontiguousarray(tiles, dtype=np.uint16)
    seg_off = np.ascontiguousarray(seg_off, dtype=np.int64)
    n = int(seg_off[-1])
    assert tiles.ndim == 2 and tiles.shape[1] >= n
    arr = (_Subgraph * len(subgraphs))(*[_subgraph(sg) for sg in subgraphs])
    s32 = np.empty(n, dtype=np.float32)
    s64 = np.empty(n, dtype=np.float64)
    feat = np.zeros((NSYM, n), dtype=np.int64) if want_symbols else None
    _check(_L().orc_draft_score(arr, len(subgraphs), _ptr(seg_off), _ptr(tiles), tiles.shape[1], flags,
                                _ptr(s32), _ptr(s64), _ptr(feat) if want_symbols else None))
    return s32, s64, feat


def topk(score, seg_off, k):
    """Per segment the k best (score descending, index ascending).  Returns (idx int32 [n_sg, k], val float32 [n_sg, k])."""
    score = np.ascontiguousarray(score, dtype=np.float32)
    seg_off = np.ascontiguousarray(seg_off, dtype=np.int64)
    n_sg = len(seg_off) - 1
    idx = np.empty((max(n_sg, 0), max(k, 0)), dtype=np.int32)
    val = np.empty((max(n_sg, 0), max(k, 0)), dtype=np.float32)
    _check(_L().orc_topk(_ptr(score), _ptr(seg_off), n_sg, k, _ptr(idx), _ptr(val)))
    return idx, val


def splitmix64_draw(seed, c):
    """The c-th output (c >= 1) of SplitMix64 started from `seed`."""
    return int(_L().orc_splitmix64_draw(seed & 0xFFFFFFFFFFFFFFFF, c & 0xFFFFFFFFFFFFFFFF))


def lse(subgraphs, seg_off, tiles, k, n_steps, seed, mutate_q16, flags=0):
    """Alg. 2 over n_steps: C_SA, PriorFilter (running k best), SchMutation.  tiles uint16 [rows, n] is not modified.

    Returns (population after the last mutation uint16 [rows, n], scores of the last scored population float32 [n],
    spec_tiles uint16 [rows, n_sg * k], spec_score float32 [n_sg, k], spec_count int32 [n_sg])."""
    pop = np.array(tiles, dtype=np.uint16, order="C", copy=True)
    seg_off = np.ascontiguousarray(seg_off, dtype=np.int64)
    n_sg, n = len(seg_off) - 1, int(seg_off[-1])
    assert pop.ndim == 2 and pop.shape[1] >= n
    arr = (_Subgraph * len(subgraphs))(*[_subgraph(sg) for sg in subgraphs])
    score = np.empty(n, dtype=np.float32)
    spec_tiles = np.zeros((pop.shape[0], n_sg * k), dtype=np.uint16)
    spec_score = np.empty((n_sg, k), dtype=np.float32)
    spec_count = np.zeros(n_sg, dtype=np.int32)
    _check(_L().orc_lse(arr, n_sg, _ptr(seg_off), _ptr(pop), pop.shape[1], pop.shape[0], flags, k, n_steps, seed & 0xFFFFFFFFFFFFFFFF,
                        mutate_q16, _ptr(score), _ptr(spec_tiles), _ptr(spec_score), _ptr(spec_count)))
    return pop, score, spec_tiles, spec_score, spec_count


def axis_space(subgraph, axis):
    """Number of schedules of one axis: ordered factorisations of its extent (over the fragment) into its levels."""
    sg = _subgraph(subgraph)
    return int(_L().orc_axis_space(C.byref(sg), axis))


def random_init(subgraphs, seg_off, rows, seed):
    """RandomInitSch: a population of schedules drawn uniformly from each subgraph's schedule space.

    Returns tiles uint16 [rows, n] (rows a subgraph does not own stay 0)."""
    seg_off = np.ascontiguousarray(seg_off, dtype=np.int64)
    n = int(seg_off[-1])
    tiles = np.zeros((rows, n), dtype=np.uint16)
    arr = (_Subgraph * len(subgraphs))(*[_subgraph(sg) for sg in subgraphs])
    _check(_L().orc_random_init(arr, len(subgraphs), _ptr(seg_off), _ptr(tiles), n, seed & 0xFFFFFFFFFFFFFFFF))
    return tiles


def moa_update(phi_s, phi_t, m):
    """Update_MoA: phi_s <- m phi_s + (1 - m) phi_t.  Returns (new phi_s float32, its bfloat16 bits uint16, the same
    update in float64)."""
    s = np.array(phi_s, dtype=np.float32, copy=True).ravel()
    t = np.ascontiguousarray(phi_t, dtype=np.float32).ravel()
    assert s.shape == t.shape
    bf = np.empty(s.size, dtype=np.uint16)
    f64 = np.empty(s.size, dtype=np.float64)
    _check(_L().orc_moa_update(_ptr(s), _ptr(t), s.size, float(m), _ptr(bf), _ptr(f64)))
    return s, bf, f64


def pacm(feat, n_stmt, flow, n_blk, weights, want_f64=True):
    """The whole Pattern-aware Transformer.  feat float32 [n_d, 8, 164], n_stmt int32 [n_d]; flow float32 [n_d, 8, 23],
    n_blk int32 [n_d]; weights as made by workloads.make_pacm_weights.  Returns (y32 float32 [n_d], y64 or None)."""
    feat = np.ascontiguousarray(feat, dtype=np.float32)
    flow = np.ascontiguousarray(flow, dtype=np.float32)
    n_stmt = np.ascontiguousarray(n_stmt, dtype=np.int32)
    n_blk = np.ascontiguousarray(n_blk, dtype=np.int32)
    n_d = feat.shape[0]
    assert feat.shape == (n_d, 8, 164) and flow.shape == (n_d, 8, 23) and n_stmt.shape == (n_d,) and n_blk.shape == (n_d,)
    keep = {}
    for k, dt in (("W1", np.uint16), ("W2", np.uint16), ("b1", np.float32), ("b2", np.float32), ("We", np.uint16), ("be", np.float32),
                  ("Wq", np.uint16), ("Wk", np.uint16), ("Wv", np.uint16), ("Wo", np.uint16), ("Wh", np.uint16), ("bh", np.float32),
                  ("wo", np.uint16)):
        keep[k] = np.ascontiguousarray(weights[k], dtype=dt)
    w = _PacmWeights(*[keep[k].ctypes.data for k in ("W1", "W2", "b1", "b2", "We", "be", "Wq", "Wk", "Wv", "Wo", "Wh", "bh", "wo")],
                     float(weights["bo"]))
    y32 = np.empty(n_d, dtype=np.float32)
    y64 = np.empty(n_d, dtype=np.float64) if want_f64 else None
    _check(_L().orc_pacm(_ptr(feat), _ptr(n_stmt), _ptr(flow), _ptr(n_blk), n_d, C.byref(w), _ptr(y32), _ptr(y64) if want_f64 else None))
    return y32, y64


def bf16_round(x):
    return np.float32(_L().orc_bf16_round(float(np.float32(x))))


def verify(feat, n_stmt, weights, want_f64=True, want_mag=False):
    """Learned-model score of every drafted candidate.

    feat float32 [n_d, max_stmt, feat_dim]; n_stmt int32 [n_d]; weights as made by workloads.make_mlp_weights.
    Returns (vscore32 float32 [n_d], vscore64 float64 [n_d] or None), and with want_mag a third array: the summed size
    of the last layer's terms per candidate (see orc_verify).
    """
    feat = np.ascontiguousarray(feat, dtype=np.float32)
    n_stmt = np.ascontiguousarray(n_stmt, dtype=np.int32)
    n_d, max_stmt, feat_dim = feat.shape
    W1 = np.ascontiguousarray(weights["W1"], dtype=np.uint16)
    W2 = np.ascontiguousarray(weights["W2"], dtype=np.uint16)
    w3 = np.ascontiguousarray(weights["w3"], dtype=np.uint16)
    b1 = np.ascontiguousarray(weights["b1"], dtype=np.float32)
    b2 = np.ascontiguousarray(weights["b2"], dtype=np.float32)
    hidden = W1.shape[0]
    assert W1.shape == (hidden, feat_dim) and W2.shape == (hidden, hidden) and w3.shape == (hidden,)
    v32 = np.empty(n_d, dtype=np.float32)
    v64 = np.empty(n_d, dtype=np.float64) if want_f64 else None
    mag = np.empty(n_d, dtype=np.float64) if want_mag else None
    _check(_L().orc_verify(_ptr(feat), _ptr(n_stmt), n_d, max_stmt, feat_dim, hidden, _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2),
                           _ptr(w3), float(weights["b3"]), _ptr(v32), _ptr(v64) if want_f64 else None,
                           _ptr(mag) if want_mag else None))
    return (v32, v64, mag) if want_mag else (v32, v64)


def verify_tolerance(v32, mag):
    """Per-candidate bound for comparing another bfloat16 evaluation of the verify model with the oracle's: 2e-2 relative,
    and never below 2^-9 of the size of the terms the score is a sum of (a score that cancels keeps the rounding steps of
    its terms)."""
    return np.maximum(2e-2 * np.abs(np.asarray(v32, np.float64)), np.asarray(mag, np.float64) / 512.0)
