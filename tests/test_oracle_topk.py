"""Pins of the oracle's selection step (PriorFilter of Alg. 2; the final selection of Alg. 1)."""
import numpy as np
import pytest

import oracle
import workloads as w


def _reference(score, seg_off, k):
    """numpy's stable sort on the negated key: first k of each segment."""
    out = []
    for s in range(len(seg_off) - 1):
        lo, hi = seg_off[s], seg_off[s + 1]
        order = np.argsort(-score[lo:hi].astype(np.float64), kind="stable")[:k]
        out.append(order + lo)
    return np.array(out, dtype=np.int32)


def test_topk_equals_stable_sort_with_many_ties():
    rng = np.random.default_rng(0)
    seg_off = np.array([0, 1000, 1003, 5000, 9000], dtype=np.int64)
    score = rng.integers(-20, 20, size=9000).astype(np.float32)      # few distinct values: ties everywhere
    for so, ks in ((seg_off, (1, 2, 3)), (np.array([0, 1000, 5000, 9000], dtype=np.int64), (64, 1000))):
        for k in ks:
            idx, val = oracle.topk(score, so, k)
            assert np.array_equal(idx, _reference(score, so, k))
            assert np.array_equal(val, score[idx])


def test_topk_special_values():
    score = np.array([0.0, -0.0, np.inf, -np.inf, 1.0, -0.0, 0.0, -1.0], dtype=np.float32)
    idx, val = oracle.topk(score, [0, 8], 8)
    # +inf first, -inf last, the four zeros in index order whatever their sign
    assert list(idx[0]) == [2, 4, 0, 1, 5, 6, 7, 3]
    with pytest.raises(oracle.OracleError):
        oracle.topk(np.array([1.0, np.nan], dtype=np.float32), [0, 2], 1)
    with pytest.raises(oracle.OracleError):
        oracle.topk(np.zeros(4, dtype=np.float32), [0, 4], 5)          # k larger than the segment
    with pytest.raises(oracle.OracleError):
        oracle.topk(np.zeros(4, dtype=np.float32), [0, 4], 0)


def test_topk_on_every_schedule_of_a_tiny_gemm():
    """Brute force: all 19,200 schedules of an 8x8x8 GEMM; annotations do not enter the draft score, so every
    tiling appears 12 times with the same score and the index tie-break decides."""
    sg = w.gemm(8, 8, 8, hw=w.toy_device())
    tiles, ann = w.enumerate_all_schedules(sg)
    n = tiles.shape[1]
    s32, s64, _ = oracle.draft_score([sg], [0, n], tiles)
    assert np.array_equal(s32.reshape(-1, 12), np.repeat(s32[::12], 12).reshape(-1, 12))
    idx, val = oracle.topk(s32, [0, n], 64)
    assert np.array_equal(idx, _reference(s32, np.array([0, n]), 64))
    best = s32.max()
    assert val[0, 0] == best and np.all(val[0, :12] == best) and list(idx[0, :12]) == sorted(idx[0, :12])
    # the best schedule by the binary64 latency is among the selected
    assert int(np.argmax(s64)) in set(idx[0])


def test_topk_is_invariant_under_a_common_scaling_of_the_peaks():
    sg1 = w.gemm(512, 512, 512)
    hw2 = w.Device(**{**sg1.hw.__dict__, "T_p": sg1.hw.T_p * 2, "T_m": sg1.hw.T_m * 2})
    sg2 = w.gemm(512, 512, 512, hw=hw2)
    tiles, _ = w.sample_population(sg1, 4096, seed=0)
    a, _, _ = oracle.draft_score([sg1], [0, 4096], tiles)
    b, _, _ = oracle.draft_score([sg2], [0, 4096], tiles)
    assert np.array_equal(oracle.topk(a, [0, 4096], 64)[0], oracle.topk(b, [0, 4096], 64)[0])
