"""Seeded random shapes through the C boundary against the oracle: the cases nobody thought of writing down.

Each test draws a fixed number of cases from a seeded generator (shapes, segment lengths, alignments, value
distributions, switches), so a failure names its seed and case and repeats exactly.  The comparisons are those of
tests/test_gpu_parity.py (check_draft, check_prior_filter, check_topk, check_verify): symbols and index lists bit for
bit, draft scores bit for bit under reference rounding and within the fused form's tolerance otherwise, verify scores
within the per-candidate tolerance.
"""
import numpy as np
import pytest

import workloads as w

import test_gpu_parity as T
from test_gpu_parity import P  # noqa: F401  (the module-scoped fixture that loads the library)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

DIMS = [8, 12, 16, 24, 32, 48, 56, 64, 96, 100, 112, 128, 192, 256, 384, 512, 768, 1000, 1024, 3072, 4096]


def _random_subgraph(rng):
    pick = lambda: int(rng.choice(DIMS))
    c = int(rng.integers(0, 6))
    if c == 0:
        return w.gemm(pick(), pick(), pick())
    if c == 1:
        return w.batched_gemm(int(rng.choice([2, 12, 16])), pick(), pick(), pick())
    if c == 2:
        return w.conv2d(int(rng.choice([1, 2, 8])), int(rng.choice([3, 16, 64, 128])), int(rng.choice([7, 14, 28, 56])),
                        int(rng.choice([7, 14, 28, 56])), int(rng.choice([16, 64, 256])), int(rng.choice([1, 3, 5])),
                        int(rng.choice([1, 3])), stride=int(rng.choice([1, 2])))
    if c == 3:
        return w.depthwise_conv2d(1, int(rng.choice([32, 96, 512])), int(rng.choice([14, 28, 56])), int(rng.choice([14, 28])), 3, 3,
                                  stride=int(rng.choice([1, 2])))
    if c == 4:
        return w.gemm(int(rng.choice([256, 1024, 4096])), int(rng.choice([256, 512, 4096])), int(rng.choice([256, 1024])),
                      dtype_bytes=2, rd_levels=3, frag=(16, 16, 16), hw=w.a100_like(2, matrix=True))
    return w.gemm(pick(), pick(), pick(), dtype_bytes=2)


@pytest.mark.parametrize("seed", [101, 102])
def test_draft_and_prior_filter_on_random_subgraphs(P, seed):
    """Mixed loop-nest classes, one to five subgraphs, segment lengths from 1 to 300,000 (one case in seven has a segment
    of more than 2^20 candidates, which takes the per-class launches), starts aligned and not, padded pitches, the ablation
    switches, with and without the symbol dump; then PriorFilter in one call on the same population."""
    rng = np.random.default_rng(seed)
    for case in range(40):
        n_sg = int(rng.choice([1, 2, 3, 5]))
        sgs = [_random_subgraph(rng) for _ in range(n_sg)]
        big = rng.random() < 0.15
        lens = [int(rng.integers(1, 300000 if big else 20000)) for _ in range(n_sg)]
        if big:
            lens[0] = int(rng.integers(1 << 20, 1300000))
        if rng.random() < 0.5:
            lens = [(L + 3) // 4 * 4 for L in lens]
        seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        slots = max(w.n_slots(s) for s in sgs)
        tiles = np.zeros((slots, int(seg[-1])), np.uint16)
        for t, sg in enumerate(sgs):
            tl, _ = w.sample_population(sg, lens[t], seed=seed * 1000 + case, stream=t)
            tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
        flags = int(rng.choice([0, 0, 1, 2, 3]))
        pad = int(rng.choice([0, 0, 3, 4]))
        symbols = bool(rng.random() < 0.5)
        k = int(min(min(lens), rng.choice([1, 16, 64, 512])))
        mode = int(rng.choice([0, 4, 8]))
        label = (seed, case, [s.name for s in sgs], lens, flags, pad, symbols, k, mode)
        try:
            T.check_draft(P, sgs, seg, tiles, flags=flags, pitch_pad=pad, symbols=symbols)
            T.check_prior_filter(P, sgs, seg, tiles, k, flags=mode)
        except AssertionError as e:
            raise AssertionError(f"case {label}: {e}") from e


@pytest.mark.parametrize("seed", [201, 202])
def test_selection_on_random_segments_and_values(P, seed):
    """All routes of the selection: k from 1 to 4096, 1 to 130 segments, lengths around every route's limits and up to three
    million, six value distributions (normal, a handful of distinct values, all equal, a narrow band, log-normal over many
    binades, infinities and signed zeros)."""
    rng = np.random.default_rng(seed)
    for case in range(60):
        k = int(rng.choice([1, 2, 7, 31, 32, 33, 64, 65, 100, 512, 1000, 4096]))
        n_sg = int(rng.choice([1, 2, 3, 8, 20, 40, 130]))
        kind = int(rng.integers(0, 4))
        lens = []
        for _ in range(n_sg):
            if kind == 0:
                L = int(rng.integers(k, max(k + 1, 9000)))
            elif kind == 1:
                L = int(rng.integers(max(k, 8000), 70000))
            elif kind == 2:
                L = int(rng.integers(max(k, 30000), 400000)) if n_sg <= 20 else int(rng.integers(k, max(k + 1, 40000)))
            else:
                L = max(k, int(rng.choice([k, k + 1, 8192, 8193, 32768, 32769, 65536, 16384 * 3 + 5])))
            lens.append(L)
        if kind == 2 and n_sg <= 3 and rng.random() < 0.3:
            lens[0] = int(rng.integers(1000000, 3000000))
        if rng.random() < 0.5:
            lens = [(L + 3) // 4 * 4 for L in lens]
        seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        n = int(seg[-1])
        dist = int(rng.integers(0, 6))
        if dist == 0:
            sc = rng.normal(size=n)
        elif dist == 1:
            sc = rng.integers(-3, 3, size=n).astype(np.float64)
        elif dist == 2:
            sc = np.full(n, -1.25)
        elif dist == 3:
            sc = -1.0 - 1e-6 * np.abs(rng.normal(size=n))
        elif dist == 4:
            sc = -np.exp(rng.normal(size=n) * 2.0)
        else:
            sc = rng.normal(size=n)
            sc[rng.integers(0, n, n // 20 + 1)] = np.inf
            sc[rng.integers(0, n, n // 3 + 1)] = 0.0
            sc[rng.integers(0, n, n // 3 + 1)] = -0.0
        try:
            T.check_topk(P, sc.astype(np.float32), seg, k)
        except AssertionError as e:
            raise AssertionError(f"case {(seed, case, k, n_sg, kind, dist, lens[:8])}: {e}") from e


def test_verify_on_random_set_sizes_and_statement_counts(P):
    """Set sizes around the tile and group sizes of the verify kernel, statement counts of every mix (uniform 0..8, all 8,
    only 0 / 1 / 8, constant over runs of 100), different weights per case, and three kinds of garbage in the ignored rows."""
    rng = np.random.default_rng(301)
    for case in range(24):
        m = w.make_mlp_weights(seed=int(rng.integers(1, 1000)))
        n_d = int(rng.choice([1, 2, 7, 8, 9, 63, 64, 65, 255, 256, 257, 1000, 2047, 2048, 2049, 4096, 5000]))
        mode = int(rng.integers(0, 4))
        if mode == 0:
            ns = rng.integers(0, 9, size=n_d)
        elif mode == 1:
            ns = np.full(n_d, 8)
        elif mode == 2:
            ns = rng.choice([0, 1, 8], size=n_d)
        else:
            ns = np.repeat(rng.integers(1, 9, size=(n_d + 99) // 100), 100)[:n_d]
        ns = ns.astype(np.int32)
        feat = w.make_statement_features(rng.integers(0, 1 << 30, size=n_d), np.maximum(ns, 1), seed=case,
                                         pad_value=float(rng.choice([0.0, 1e30, -7.5])))
        for c in np.flatnonzero(ns == 0):
            feat[c] = 3.0
        try:
            T.check_verify(P, feat, ns, m)
        except AssertionError as e:
            raise AssertionError(f"case {(case, n_d, mode)}: {e}") from e
