"""Pins of the oracle's whole Pattern-aware Transformer (Sec. 4.2: statement branch, self-attention over temporal dataflow
blocks, concatenation, linear head).

The paper's figure with the dimensions is lost: the shape of the model is a reading ("parity unpinned" by the paper).
Pinned here is what the text and the mathematics fix: hand-sized cases worked out by hand, the reduction of the statement
branch plus an identity head to the already pinned statement model, the invariances of sum pooling and of attention
without positions, the limits of the softmax, and the agreement of the two precisions.
"""
import numpy as np
import pytest

import oracle
import workloads as w

bf = w.f32_to_bf16_bits


def zero_weights():
    z = lambda *s: bf(np.zeros(s, np.float32))
    return {"W1": z(256, 164), "b1": np.zeros(256, np.float32), "W2": z(256, 256), "b2": np.zeros(256, np.float32),
            "We": z(64, 23), "be": np.zeros(64, np.float32), "Wq": z(64, 64), "Wk": z(64, 64), "Wv": z(64, 64), "Wo": z(64, 64),
            "Wh": z(256, 320), "bh": np.zeros(256, np.float32), "wo": z(256), "bo": 0.0}


def put(m, name, entries):
    a = w.bf16_bits_to_f32(m[name]).copy()
    for idx, v in entries.items():
        a[idx] = v
    m[name] = bf(a)


def inputs(n_d, n_stmt, n_blk, seed=0):
    ids = np.arange(n_d) * 13 + 1
    return (w.make_statement_features(ids, n_stmt, seed=seed), np.asarray(n_stmt, np.int32),
            w.make_flow_features(ids, n_blk, seed=seed), np.asarray(n_blk, np.int32))


def test_no_statements_and_no_blocks_leave_the_head_bias_path():
    m = w.make_pacm_weights(seed=2)
    feat, n_stmt, flow, n_blk = inputs(3, [0, 0, 0], [0, 0, 0])
    y32, y64 = oracle.pacm(feat, n_stmt, flow, n_blk, m)
    wo = w.bf16_bits_to_f32(m["wo"]).astype(np.float64)
    want = float(wo @ np.maximum(m["bh"].astype(np.float64), 0.0) + m["bo"])
    assert np.allclose(y64, want, rtol=1e-12)
    assert np.allclose(y32, want, rtol=1e-2)


def test_hand_sized_dataflow_branch():
    """Embedding e = (d0, d1); Wq = Wk = 0 make the attention uniform; Wv = I, Wo = 2 I on two units:
    o_i = mean of e, z_i = e_i + 2 mean, v_d = sum_i z_i = 3 sum_i e_i.  Head: g0 = v_d[0] - v_d[1] + 1, y = 2 g0 - 0.5."""
    m = zero_weights()
    put(m, "We", {(0, 0): 1.0, (1, 1): 1.0})
    put(m, "Wv", {(0, 0): 1.0, (1, 1): 1.0})
    put(m, "Wo", {(0, 0): 2.0, (1, 1): 2.0})
    put(m, "Wh", {(0, 256): 1.0, (0, 257): -1.0})
    m["bh"][0] = 1.0
    put(m, "wo", {0: 2.0})
    m["bo"] = -0.5
    flow = np.zeros((2, 8, 23), np.float32)
    flow[0, 0, :2], flow[0, 1, :2], flow[0, 2, :2] = (1, 2), (3, 0), (4, 1)      # sum e = (8, 3): v_d = (24, 9): g0 = 16: y = 31.5
    flow[1, 0, :2] = (5, 1)                                                      # one block: v_d = (15, 3): g0 = 13: y = 25.5
    flow[1, 1, :2] = (100, -7)                                                   # beyond n_blk: ignored
    y32, y64 = oracle.pacm(np.zeros((2, 8, 164), np.float32), [0, 0], flow, [3, 1], m)
    assert list(y32) == [31.5, 25.5] and np.allclose(y64, [31.5, 25.5], rtol=1e-14)   # (thirds are not binary fractions)


def test_sharp_attention_picks_one_block():
    """q . k / 8 = 64 e0_i e0_j: with e0 in {0, 1} the rows whose e0 is 1 attend (almost) only to blocks whose e0 is 1."""
    m = zero_weights()
    put(m, "We", {(0, 0): 1.0, (1, 1): 1.0})
    put(m, "Wq", {(0, 0): 16.0})
    put(m, "Wk", {(0, 0): 32.0})
    put(m, "Wv", {(1, 1): 1.0})
    put(m, "Wo", {(1, 1): 1.0})
    put(m, "Wh", {(0, 257): 1.0})
    put(m, "wo", {0: 1.0})
    flow = np.zeros((1, 8, 23), np.float32)
    flow[0, 0, :2], flow[0, 1, :2] = (1, 7), (0, 3)
    # block 0 (e0 = 1): scores (64, 0): attends to itself: o = 7; block 1 (e0 = 0): scores (0, 0): uniform: o = 5
    # v_d[1] = (7 + 7) + (3 + 5) = 22
    y32, y64 = oracle.pacm(np.zeros((1, 8, 164), np.float32), [0], flow, [2], m)
    assert abs(y64[0] - 22.0) < 1e-12 * 22 + 2 * np.exp(-64.0) * 10
    assert y32[0] == 22.0


def test_statement_branch_with_an_identity_head_is_the_statement_model():
    """Wh = [I | 0], bh = 0, wo = w3: y = w3 . v_s + bo, the summed statement model without its per-statement bias
    (up to the bfloat16 rounding of v_s)."""
    mlp = w.make_mlp_weights(seed=1)
    m = zero_weights()
    for k in ("W1", "b1", "W2", "b2"):
        m[k] = mlp[k]
    m["Wh"] = bf(np.concatenate([np.eye(256, dtype=np.float32), np.zeros((256, 64), np.float32)], axis=1))
    m["wo"], m["bo"] = mlp["w3"], 0.25
    n_stmt = np.array([1, 3, 8, 5, 0, 2], np.int32)
    feat, n_stmt, flow, n_blk = inputs(6, n_stmt, [0] * 6, seed=4)
    y32, y64 = oracle.pacm(feat, n_stmt, flow, n_blk, m)
    v32, v64 = oracle.verify(feat, n_stmt, mlp)
    want = v64 - n_stmt * mlp["b3"] + 0.25
    assert np.allclose(y64, want, rtol=1e-9, atol=1e-9)
    assert np.all(np.abs(y32 - want) <= 2e-2 * np.maximum(np.abs(want), 1e-2 * np.abs(want).max()))


def test_order_of_statements_and_of_blocks_does_not_matter():
    m = w.make_pacm_weights(seed=1)
    n_stmt, n_blk = [8, 5, 3], [8, 4, 6]
    feat, n_stmt, flow, n_blk = inputs(3, n_stmt, n_blk, seed=7)
    y32, y64 = oracle.pacm(feat, n_stmt, flow, n_blk, m)
    f2, d2 = feat.copy(), flow.copy()
    for c in range(3):
        f2[c, :n_stmt[c]] = feat[c, :n_stmt[c]][::-1]
        d2[c, :n_blk[c]] = np.roll(flow[c, :n_blk[c]], 2, axis=0)
    z32, z64 = oracle.pacm(f2, n_stmt, d2, n_blk, m)
    assert np.allclose(z64, y64, rtol=1e-11)
    assert np.allclose(z32, y32, rtol=2e-2)
    # rows beyond the counts are ignored whatever they hold
    f3, d3 = feat.copy(), flow.copy()
    for c in range(3):
        f3[c, n_stmt[c]:] = 1e30
        d3[c, n_blk[c]:] = -1e30
    w32, w64 = oracle.pacm(f3, n_stmt, d3, n_blk, m)
    assert np.array_equal(w32, y32) and np.array_equal(w64, y64)


def test_the_two_precisions_agree_and_the_branches_matter():
    m = w.make_pacm_weights(seed=1)
    rng = np.random.default_rng(5)
    n_d = 40
    feat, n_stmt, flow, n_blk = inputs(n_d, rng.integers(0, 9, n_d), rng.integers(0, 9, n_d), seed=9)
    y32, y64 = oracle.pacm(feat, n_stmt, flow, n_blk, m)
    # bfloat16 operands (the pooled vectors among them, whose entries reach the tens) against no rounding at all: within
    # one percent of the output range
    tol = np.full(n_d, 1e-2 * np.abs(y64).max())
    assert np.all(np.abs(y32 - y64) <= tol)
    # dropping either branch's input changes the prediction
    a32, _ = oracle.pacm(feat, np.zeros(n_d, np.int32), flow, n_blk, m)
    b32, _ = oracle.pacm(feat, n_stmt, flow, np.zeros(n_d, np.int32), m)
    assert np.abs(a32 - y32).max() > 10 * tol.max() or np.abs(a32 - y32).mean() > tol.mean()
    assert np.abs(b32 - y32)[n_blk > 0].min() > 0


def test_bad_counts_are_refused():
    m = w.make_pacm_weights(seed=1)
    feat, n_stmt, flow, n_blk = inputs(2, [1, 1], [1, 1])
    with pytest.raises(oracle.OracleError):
        oracle.pacm(feat, [9, 1], flow, n_blk, m)
    with pytest.raises(oracle.OracleError):
        oracle.pacm(feat, n_stmt, flow, [1, -1], m)


def test_the_absolute_term_of_the_comparison_bound_is_sized_from_the_two_precisions():
    """The GPU tests allow |g - o| <= 2e-2 |o| + 5e-3 max|o| between the kernels and this oracle.  The absolute term covers
    what a 2e-2 relative bound cannot: a pooled vector entry that lands on the other side of a bfloat16 rounding boundary
    moves the head's output by an amount that does not depend on the output's own size.  The oracle's own two evaluations
    of the same inputs (bfloat16 operands with binary32 accumulation; binary64 without any rounding of operands) show the
    size of that effect: on the GPU tests' kind of inputs their largest gap is just under one hundredth of the output
    range.  The term allows the kernels between a quarter of that gap and the whole of it (they round the same operands
    as the oracle's first evaluation, so they sit closer to it than the second does): not loose enough to hide a wrong
    sign or a dropped block, as the second half shows."""
    m = w.make_pacm_weights(seed=1)
    rng = np.random.default_rng(5)
    n_d = 600
    n_stmt = rng.integers(0, 9, size=n_d).astype(np.int32)
    n_blk = rng.integers(0, 9, size=n_d).astype(np.int32)
    feat, n_stmt, flow, n_blk = inputs(n_d, n_stmt, n_blk, seed=3)
    y32, y64 = oracle.pacm(feat, n_stmt, flow, n_blk, m)
    span = float(np.abs(y32).max())
    gap = float(np.abs(y32 - y64).max())
    term = 5e-3 * span
    assert term <= gap <= 4 * term, (gap, term)
    tol = 2e-2 * np.abs(y32) + term
    # mistakes the bound must still see: one dataflow block too few, and the head's bias with the wrong sign
    fewer, _ = oracle.pacm(feat, n_stmt, flow, np.maximum(n_blk - 1, 0), m)
    assert (np.abs(fewer - y32) > tol)[n_blk >= 1].mean() > 0.9
    flipped = dict(m)
    flipped["bo"] = -m["bo"] if abs(m["bo"]) > 0.05 else m["bo"] + 1.0
    wrong, _ = oracle.pacm(feat, n_stmt, flow, n_blk, flipped)
    assert (np.abs(wrong - y32) > tol).mean() > 0.9
