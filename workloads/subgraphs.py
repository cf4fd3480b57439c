"""Loop-nest descriptors of the subgraphs whose schedules are explored.

A subgraph is one tiled reduction statement  O[sp] (+)= f(In_0[..], In_1[..]):
`n_sp` spatial axes followed by `n_rd` reduction axes, each buffer indexed by
affine expressions of the axis variables.  This replaces the sketch that
`GenerateSketch` would produce inside a tensor compiler (Alg. 2): it is the
fixed part of the input; the tile factors are the variable part.

`Device` is the device abstraction `d` of Alg. 1 / Alg. 2, i.e. the constants
named in the "Hardware-aware Penalty" paragraph (Sec. 4.1):
T_p, T_m, m_l0, m_l1, pu_l1, n_l1, pu_l2, n_l2.  These describe the device the
schedules are *tuned for*, not the GPU that runs the scoring.
"""
from dataclasses import dataclass, field
from typing import Tuple


@dataclass(frozen=True)
class Device:
    T_p: float      # theoretical peak compute, flop/s
    T_m: float      # theoretical peak bandwidth of the lowest storage level, byte/s
    m_l0: int       # L0 (register) allocation limit per thread, elements
    m_l1: int       # L1 (shared memory) allocation limit per block, bytes
    pu_l1: int      # L1 scheduling blocks that can be active at once
    n_l1: int       # scheduling size within a block (warp size)
    pu_l2: int      # L2-level parallel units (SMs / CUs)
    n_l2: int       # memory transaction length, elements of the subgraph's dtype


# One index expression per buffer dimension: ((axis, coef), ...), at most 2 terms.
Dim = Tuple[Tuple[int, int], ...]


@dataclass(frozen=True)
class Buffer:
    dims: Tuple[Dim, ...]   # row-major, last dimension contiguous; at most 4 dims


@dataclass(frozen=True)
class Subgraph:
    name: str
    n_sp: int                       # spatial axes (<= 4)
    n_rd: int                       # reduction axes (<= 3)
    extent: Tuple[int, ...]         # spatial extents, then reduction extents
    sp_levels: int                  # split levels of every spatial axis (4)
    rd_levels: int                  # split levels of every reduction axis (2 or 3)
    dtype_bytes: int
    frag: Tuple[int, int, int]      # (0,0,0) or the matrix-fragment shape, e.g. (16,16,16)
    inputs: Tuple[Buffer, ...]      # 1 or 2 input buffers
    out: Buffer
    hw: Device
    axis_names: Tuple[str, ...] = field(default=(), compare=False)


def n_slots(sg: Subgraph) -> int:
    """Tile-factor slots of one candidate: axis-major, outermost level first."""
    return sg.n_sp * sg.sp_levels + sg.n_rd * sg.rd_levels


def a100_like(dtype_bytes: int, matrix: bool = False) -> Device:
    """Public datasheet figures of the paper's main platform (Sec. 5, "Platforms")."""
    return Device(
        T_p=312e12 if matrix else 19.5e12,
        T_m=1.555e12,
        m_l0=255,
        m_l1=49152,
        pu_l1=4,
        n_l1=32,
        pu_l2=108,
        n_l2=32 // dtype_bytes,
    )


def toy_device() -> Device:
    """Tiny round numbers for hand-computed examples."""
    return Device(T_p=1024.0, T_m=256.0, m_l0=8, m_l1=64, pu_l1=2, n_l1=4, pu_l2=4, n_l2=4)


def _d(*terms) -> Dim:
    return tuple(terms)


def gemm(M, N, K, dtype_bytes=4, hw=None, sp_levels=4, rd_levels=2, frag=(0, 0, 0), name=None):
    """C[i,j] += A[i,k] * B[k,j]; axes i=0, j=1 (spatial), k=2 (reduction)."""
    hw = hw or a100_like(dtype_bytes, matrix=frag != (0, 0, 0))
    A = Buffer((_d((0, 1)), _d((2, 1))))
    B = Buffer((_d((2, 1)), _d((1, 1))))
    C = Buffer((_d((0, 1)), _d((1, 1))))
    return Subgraph(name or f"gemm_{M}x{N}x{K}", 2, 1, (M, N, K), sp_levels, rd_levels,
                    dtype_bytes, tuple(frag), (A, B), C, hw, ("i", "j", "k"))


def batched_gemm(Bt, M, N, K, dtype_bytes=4, hw=None, sp_levels=4, rd_levels=2, frag=(0, 0, 0), name=None):
    """C[b,i,j] += A[b,i,k] * B[b,k,j]; axes b=0, i=1, j=2 (spatial), k=3 (reduction)."""
    hw = hw or a100_like(dtype_bytes, matrix=frag != (0, 0, 0))
    A = Buffer((_d((0, 1)), _d((1, 1)), _d((3, 1))))
    B = Buffer((_d((0, 1)), _d((3, 1)), _d((2, 1))))
    C = Buffer((_d((0, 1)), _d((1, 1)), _d((2, 1))))
    return Subgraph(name or f"bgemm_{Bt}x{M}x{N}x{K}", 3, 1, (Bt, M, N, K), sp_levels, rd_levels,
                    dtype_bytes, tuple(frag), (A, B), C, hw, ("b", "i", "j", "k"))


def conv2d(N, C, H, W, K, R, S, stride=1, pad=1, dtype_bytes=4, hw=None, name=None):
    """O[n,k,h,w] += I[n,c,h*stride+r,w*stride+s] * Wt[k,c,r,s] (implicit-GEMM nest).

    Spatial axes n=0,k=1,h=2,w=3 over the OUTPUT extents; reduction c=4,r=5,s=6.
    """
    hw = hw or a100_like(dtype_bytes)
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    I = Buffer((_d((0, 1)), _d((4, 1)), _d((2, stride), (5, 1)), _d((3, stride), (6, 1))))
    Wt = Buffer((_d((1, 1)), _d((4, 1)), _d((5, 1)), _d((6, 1))))
    O = Buffer((_d((0, 1)), _d((1, 1)), _d((2, 1)), _d((3, 1))))
    return Subgraph(name or f"conv2d_n{N}c{C}h{H}w{W}k{K}r{R}s{S}", 4, 3, (N, K, Ho, Wo, C, R, S), 4, 2,
                    dtype_bytes, (0, 0, 0), (I, Wt), O, hw, ("n", "k", "h", "w", "c", "r", "s"))


def depthwise_conv2d(N, C, H, W, R, S, stride=1, pad=1, dtype_bytes=4, hw=None, name=None):
    """O[n,c,h,w] += I[n,c,h*stride+r,w*stride+s] * Wt[c,r,s]; reduction r=4, s=5."""
    hw = hw or a100_like(dtype_bytes)
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    I = Buffer((_d((0, 1)), _d((1, 1)), _d((2, stride), (4, 1)), _d((3, stride), (5, 1))))
    Wt = Buffer((_d((1, 1)), _d((4, 1)), _d((5, 1))))
    O = Buffer((_d((0, 1)), _d((1, 1)), _d((2, 1)), _d((3, 1))))
    return Subgraph(name or f"dwconv_n{N}c{C}h{H}w{W}r{R}s{S}", 4, 2, (N, C, Ho, Wo, R, S), 4, 2,
                    dtype_bytes, (0, 0, 0), (I, Wt), O, hw, ("n", "c", "h", "w", "r", "s"))
