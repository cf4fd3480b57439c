"""Candidate schedules: multi-level tile factorisations plus annotations.

A candidate assigns to every axis of a subgraph an ordered factorisation of
its extent (one factor per split level, outermost first) and picks an unroll
factor and a vector width: the "tile sizes, unroll factors" that span the
tuning space (Sec. 2.1).  Populations are stored structure-of-arrays:

    tiles[slot, c]   uint16   slot = axis-major, then level (outermost first)
    ann[c]           uint16   unroll_idx | (vec_idx << 8)

They stand in for `RandomInitSch` (Alg. 2): each factorisation is drawn
uniformly from all ordered factorisations of the extent.
"""
import itertools
from functools import lru_cache
from math import comb

import numpy as np

from .rng import hash_u64
from .subgraphs import Subgraph, n_slots

UNROLL_VALUES = (0, 16, 64, 512)
VECTOR_VALUES = (1, 2, 4)


def _divisors(n):
    return [d for d in range(1, n + 1) if n % d == 0]


@lru_cache(maxsize=None)
def _ordered_factorizations(n, levels):
    if levels == 1:
        return ((n,),)
    out = []
    for d in _divisors(n):
        for rest in _ordered_factorizations(n // d, levels - 1):
            out.append((d,) + rest)
    return tuple(out)


def ordered_factorizations(n, levels):
    """All (f_0..f_{levels-1}) of positive ints with product n, lexicographic; uint16 [count, levels]."""
    return np.array(_ordered_factorizations(int(n), int(levels)), dtype=np.uint16).reshape(-1, levels)


def count_ordered_factorizations(n, levels):
    """Closed form: prod over prime powers p^e of C(e + levels - 1, levels - 1)."""
    total, p = 1, 2
    while n > 1:
        e = 0
        while n % p == 0:
            n //= p
            e += 1
        if e:
            total *= comb(e + levels - 1, levels - 1)
        p += 1
    return total


def _frag_of_axis(sg: Subgraph, axis: int) -> int:
    """Fragment size that constrains the innermost factor of `axis` (1 = unconstrained)."""
    if sg.frag == (0, 0, 0):
        return 1
    if axis == sg.n_sp - 2:
        return sg.frag[0]
    if axis == sg.n_sp - 1:
        return sg.frag[1]
    if axis == sg.n_sp + sg.n_rd - 1:
        return sg.frag[2]
    return 1


def axis_tables(sg: Subgraph):
    """Per axis, the table [count, levels] of admissible ordered factorisations.

    In fragment mode the innermost factor of the two innermost spatial axes and
    of the last reduction axis is a multiple of the fragment size: the table is
    the factorisations of extent/frag with the last column scaled by frag.
    """
    tables = []
    for a in range(sg.n_sp + sg.n_rd):
        levels = sg.sp_levels if a < sg.n_sp else sg.rd_levels
        f = _frag_of_axis(sg, a)
        if sg.extent[a] % f:
            raise ValueError(f"extent {sg.extent[a]} of axis {a} is not a multiple of fragment {f}")
        t = ordered_factorizations(sg.extent[a] // f, levels).astype(np.uint32)
        t[:, -1] *= f
        if t.max() > 0xFFFF:
            raise ValueError("tile factor does not fit uint16")
        tables.append(t.astype(np.uint16))
    return tables


def sample_population(sg: Subgraph, n: int, seed: int, stream: int = 0, first: int = 0):
    """Draw candidates first..first+n-1 of the population keyed (seed, stream).

    Returns (tiles uint16 [slots, n], ann uint16 [n]).  Candidate c depends only
    on (seed, stream, c), so any slice of a population can be regenerated alone.
    """
    cand = np.arange(first, first + n, dtype=np.uint64)
    tiles = np.empty((n_slots(sg), n), dtype=np.uint16)
    slot = 0
    for a, table in enumerate(axis_tables(sg)):
        pick = (hash_u64(seed, stream * 64 + a, cand) % np.uint64(len(table))).astype(np.int64)
        levels = table.shape[1]
        tiles[slot:slot + levels, :] = table[pick].T
        slot += levels
    unroll = (hash_u64(seed, stream * 64 + 32, cand) % np.uint64(len(UNROLL_VALUES))).astype(np.uint16)
    vec = (hash_u64(seed, stream * 64 + 33, cand) % np.uint64(len(VECTOR_VALUES))).astype(np.uint16)
    ann = unroll | (vec << np.uint16(8))
    return tiles, ann


def enumerate_all_schedules(sg: Subgraph):
    """Every schedule of a (tiny) subgraph: all tilings x all annotations.

    Order: lexicographic in (axis 0 table index, ..., last axis table index,
    unroll_idx, vec_idx).  Returns (tiles uint16 [slots, n], ann uint16 [n]).
    """
    tables = axis_tables(sg)
    ranges = [range(len(t)) for t in tables] + [range(len(UNROLL_VALUES)), range(len(VECTOR_VALUES))]
    combos = np.array(list(itertools.product(*ranges)), dtype=np.int64)
    n = len(combos)
    tiles = np.empty((n_slots(sg), n), dtype=np.uint16)
    slot = 0
    for a, table in enumerate(tables):
        levels = table.shape[1]
        tiles[slot:slot + levels, :] = table[combos[:, a]].T
        slot += levels
    ann = (combos[:, -2] | (combos[:, -1] << 8)).astype(np.uint16)
    return tiles, ann
