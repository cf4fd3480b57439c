"""Pins of the oracle's learned-model branch: linear layers on statement features, then a sum over
statements (Sec. 4.2, Pattern-aware Transformer), in bfloat16 with binary32 accumulation."""
import numpy as np
import torch

import oracle
import workloads as w


def _zero_weights():
    m = w.make_mlp_weights(seed=1)
    for k in ("W1", "W2", "w3"):
        m[k] = np.zeros_like(m[k])
    for k in ("b1", "b2"):
        m[k] = np.zeros_like(m[k])
    return m


def test_bf16_rounding_matches_torch_and_ties_go_to_even():
    xs = np.concatenate([np.random.default_rng(0).normal(size=2000).astype(np.float32) * 50,
                         np.array([1.00390625, 1.01171875, 0.0, -0.0, 65504.0, 1e-40], dtype=np.float32)])
    want = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.bf16_round(x) for x in xs], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_zero_weights_give_n_stmt_times_b3():
    m = _zero_weights()
    m["b3"] = 0.375
    n_stmt = np.array([0, 1, 3, 8, 5], dtype=np.int32)
    feat = w.make_statement_features(np.arange(5), n_stmt)
    v32, v64 = oracle.verify(feat, n_stmt, m)
    assert np.array_equal(v32, (n_stmt * 0.375).astype(np.float32)) and np.array_equal(v64, n_stmt * 0.375)


def test_padded_rows_do_not_contribute():
    m = w.make_mlp_weights(seed=1)
    n_stmt = np.array([3, 8, 1, 5], dtype=np.int32)
    clean = w.make_statement_features(np.arange(4), n_stmt)
    dirty = w.make_statement_features(np.arange(4), n_stmt, pad_value=1e6)
    a, _ = oracle.verify(clean, n_stmt, m)
    b, _ = oracle.verify(dirty, n_stmt, m)
    assert np.array_equal(a, b)
    # and a statement more changes the result by that statement's output
    c, _ = oracle.verify(dirty, np.array([4, 8, 2, 6], dtype=np.int32), m)
    assert not np.any(c == a)[()] or c[1] == a[1]


def test_hand_sized_network():
    """feat_dim 2, hidden 2, exact small integers: y = w3 . relu(W2 relu(W1 x + b1) + b2) + b3."""
    bf = w.f32_to_bf16_bits
    m = {"W1": bf(np.array([[1, -1], [2, 0]], np.float32)), "b1": np.array([0, -3], np.float32),
         "W2": bf(np.array([[1, 1], [-1, 2]], np.float32)), "b2": np.array([1, 0], np.float32),
         "w3": bf(np.array([2, -1], np.float32)), "b3": 0.5}
    feat = np.array([[[3, 1], [1, 5]], [[2, 2], [9, 9]]], np.float32)
    # c0 s0: x=(3,1): h1=relu(2, 3)=(2,3); h2=relu(5+1, -2+6)=(6,4); y=12-4+.5=8.5
    # c0 s1: x=(1,5): h1=relu(-4,-1)=(0,0); h2=relu(1,0)=(1,0); y=2.5          -> 11.0
    # c1 s0: x=(2,2): h1=relu(0, 1)=(0,1); h2=relu(2, 2)=(2,2); y=4-2+.5=2.5   (only one valid statement)
    v32, v64 = oracle.verify(feat, np.array([2, 1], np.int32), m)
    assert list(v32) == [11.0, 2.5] and list(v64) == [11.0, 2.5]


def test_against_torch_linear_layers():
    """Library cross-check: torch CPU fp32 linear layers on the same bf16-rounded values."""
    m = w.make_mlp_weights(seed=1)
    n_stmt = np.array([3, 4, 5, 6, 7, 8, 1, 2] * 4, dtype=np.int32)
    feat = w.make_statement_features(np.arange(32) * 977, n_stmt)
    v32, v64 = oracle.verify(feat, n_stmt, m)

    def bf(t):
        return t.to(torch.bfloat16).to(torch.float64)

    W1 = torch.from_numpy(w.bf16_bits_to_f32(m["W1"])).double()
    W2 = torch.from_numpy(w.bf16_bits_to_f32(m["W2"])).double()
    w3 = torch.from_numpy(w.bf16_bits_to_f32(m["w3"])).double()
    b1, b2 = torch.from_numpy(m["b1"]).double(), torch.from_numpy(m["b2"]).double()
    x = torch.from_numpy(feat)
    # bf16 path, with fp64 accumulation in place of the oracle's ordered fp32 one
    h1 = bf(torch.relu(torch.nn.functional.linear(bf(x), W1, b1)).float())
    h2 = bf(torch.relu(torch.nn.functional.linear(h1, W2, b2)).float())
    y = torch.nn.functional.linear(h2, w3[None, :]).squeeze(-1) + m["b3"]
    mask = torch.arange(8)[None, :] < torch.from_numpy(n_stmt)[:, None]
    want = (y * mask).sum(dim=1).numpy()
    scale = np.abs(want).max()
    assert np.all(np.abs(v32 - want) <= 2e-3 * np.maximum(np.abs(want), 1e-3 * scale))
    # unrounded fp64 network against the oracle's fp64 shadow
    g1 = torch.relu(torch.nn.functional.linear(x.double(), W1, b1))
    g2 = torch.relu(torch.nn.functional.linear(g1, W2, b2))
    y64 = torch.nn.functional.linear(g2, w3[None, :]).squeeze(-1) + m["b3"]
    want64 = (y64 * mask).sum(dim=1).numpy()
    assert np.allclose(v64, want64, rtol=1e-12, atol=1e-12 * scale)
    # bf16 rounding moves the result by about 2^-8 relative, far inside the 2e-2 parity tolerance
    assert np.all(np.abs(v32 - v64) <= 2e-2 * np.maximum(np.abs(v64), 1e-3 * scale))


# ---- the bound used when another bfloat16 evaluation (the GPU's) is compared with the oracle's ---------------------------

def test_term_size_on_the_hand_sized_network_and_on_zero_weights():
    bf = w.f32_to_bf16_bits
    m = {"W1": bf(np.array([[1, -1], [2, 0]], np.float32)), "b1": np.array([0, -3], np.float32),
         "W2": bf(np.array([[1, 1], [-1, 2]], np.float32)), "b2": np.array([1, 0], np.float32),
         "w3": bf(np.array([2, -1], np.float32)), "b3": 0.5}
    feat = np.array([[[3, 1], [1, 5]], [[2, 2], [9, 9]]], np.float32)
    # h2 = (6,4), (1,0) | (2,2): sizes 12 + 4 + .5, 2 + 0 + .5 | 4 + 2 + .5
    _, _, mag = oracle.verify(feat, np.array([2, 1], np.int32), m, want_mag=True)
    assert list(mag) == [19.0, 6.5]
    z = _zero_weights()
    z["b3"] = -0.375
    n_stmt = np.array([0, 1, 8], np.int32)
    _, _, mag = oracle.verify(w.make_statement_features(np.arange(3), n_stmt), n_stmt, z, want_mag=True)
    assert list(mag) == [0.0, 0.375, 3.0]


def _bf16(x):
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32).view(np.float32)


def _network_in_another_order(feat, n_stmt, m, seed):
    """The same bfloat16 network with the products of a layer accumulated in binary32 in another order: depth blocks of 16
    (a matrix-core step), each summed by the library's own routine, the blocks added in a shuffled order."""
    W1, W2, w3 = (w.bf16_bits_to_f32(m[k]) for k in ("W1", "W2", "w3"))

    def layer(A, B):
        pad = (-A.shape[1]) % 16
        A, B = np.pad(A, ((0, 0), (0, pad))), np.pad(B, ((0, 0), (0, pad)))
        steps = np.arange(A.shape[1] // 16)
        np.random.default_rng(seed).shuffle(steps)
        acc = np.zeros((A.shape[0], B.shape[0]), np.float32)
        for s in steps:
            acc = acc + (A[:, 16 * s:16 * s + 16] @ B[:, 16 * s:16 * s + 16].T).astype(np.float32)
        return acc

    x = _bf16(feat.reshape(-1, feat.shape[-1]))
    h1 = _bf16(np.maximum(layer(x, W1) + m["b1"], 0))
    h2 = _bf16(np.maximum(layer(h1, W2) + m["b2"], 0))
    y = ((h2 * w3).sum(1, dtype=np.float32) + np.float32(m["b3"])).reshape(len(n_stmt), -1)
    return (y * (np.arange(y.shape[1])[None, :] < n_stmt[:, None])).sum(1, dtype=np.float32)


def test_the_comparison_bound_covers_reordered_accumulation_and_still_sees_mistakes():
    """oracle.verify_tolerance (2e-2 relative, at least 2^-9 of the summed term sizes) is what the GPU tests allow between the
    kernel and the oracle.  On those tests' inputs: (i) evaluations that differ from the oracle only in the order of the
    binary32 accumulation stay within a quarter of it, and so does the oracle's binary64 shadow within the whole of it:
    the bound is not tight by accident; (ii) a dropped statement row, a statement too many, or a sign error in the last
    bias exceed it for nearly every candidate: the bound is not loose either."""
    m = w.make_mlp_weights(seed=1)
    rng = np.random.default_rng(3)
    n_d = 1500
    n_stmt = rng.integers(0, 9, size=n_d).astype(np.int32)
    feat = w.make_statement_features(np.arange(n_d) * 31 + 5, n_stmt)
    o32, o64, mag = oracle.verify(feat, n_stmt, m, want_mag=True)
    tol = oracle.verify_tolerance(o32, mag)
    assert np.array_equal(tol[n_stmt == 0], np.zeros((n_stmt == 0).sum()))
    worst = 0.0
    for seed in (1, 2, 3):
        other = _network_in_another_order(feat, n_stmt, m, seed)
        assert np.all(np.abs(other - o32) <= tol / 4)
        worst = max(worst, float((np.abs(other - o32)[n_stmt > 0] / tol[n_stmt > 0]).max()))
    assert worst > 1e-3                                        # the orders do differ: the check above is not vacuous
    assert np.all(np.abs(o64 - o32) <= tol)
    # mistakes
    live = n_stmt >= 2
    fewer, _ = oracle.verify(feat, np.maximum(n_stmt - 1, 0), m)
    assert (np.abs(fewer - o32) > tol)[live].mean() > 0.97
    dirty = w.make_statement_features(np.arange(n_d) * 31 + 5, n_stmt, pad_value=12.0)    # padded rows hold something
    more, _ = oracle.verify(dirty, np.minimum(n_stmt + 1, 8), m)
    assert (np.abs(more - o32) > tol)[(n_stmt >= 1) & (n_stmt < 8)].mean() > 0.97
    flipped = dict(m)
    flipped["b3"] = -m["b3"]
    wrong, _ = oracle.verify(feat, n_stmt, flipped)
    if abs(m["b3"]) > 0.02:
        assert (np.abs(wrong - o32) > tol)[n_stmt >= 4].mean() > 0.5
