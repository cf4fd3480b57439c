"""Pins of the CPU oracle's Symbol-based Analyzer against what the paper and arithmetic fix.

None of these tests touches the GPU library.  Each is chosen so that a plausible
mistake in the oracle (a dropped term, a swapped operand, a wrong level mapping,
a transposed access) breaks at least one of them.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as w

ROOMY = w.Device(T_p=1024.0, T_m=256.0, m_l0=1024, m_l1=8192, pu_l1=2, n_l1=4, pu_l2=4, n_l2=4)


def _build(desc):
    d = dict(desc)
    kind = d.pop("kind")
    hw = {"toy": w.toy_device(), "roomy": ROOMY}[d.pop("device")]
    if kind == "gemm":
        return w.gemm(d["M"], d["N"], d["K"], dtype_bytes=d["dtype_bytes"], hw=hw, rd_levels=d["rd_levels"], frag=tuple(d["frag"]))
    if kind == "conv2d":
        return w.conv2d(d["N"], d["C"], d["H"], d["W"], d["K"], d["R"], d["S"], stride=d["stride"], pad=d["pad"],
                        dtype_bytes=d["dtype_bytes"], hw=hw)
    raise ValueError(kind)


def _examples(golden_dir):
    with open(os.path.join(golden_dir, "sa_worked_examples.json")) as f:
        return json.load(f)["examples"]


def test_worked_examples_symbols_terms_and_latency(golden_dir):
    """Hand-computed examples (tests/golden/sa_worked_examples.json): Table 2, the penalty paragraph and Eq. 1."""
    for ex in _examples(golden_dir):
        sg = _build(ex["subgraph"])
        sym, t64, t32 = oracle.analyze_candidate(sg, ex["factors"])
        assert sym == ex["symbols"], ex["name"]
        for name, frac in ex["terms"].items():
            want = float(Fraction(frac))
            assert t64[name] == pytest.approx(want, rel=1e-14), (ex["name"], name)
            assert float(t32[name]) == pytest.approx(want, rel=1e-6), (ex["name"], name)
        want = float(Fraction(ex["L_total"]))
        assert t64["Ltotal"] == pytest.approx(want, rel=1e-14), ex["name"]
        assert float(t32["Ltotal"]) == pytest.approx(want, rel=1e-6), ex["name"]
        s32, s64, _ = oracle.draft_score([sg], [0, 1], np.array(ex["factors"], dtype=np.uint16)[:, None])
        assert s64[0] == -t64["Ltotal"] and s32[0] == -t32["Ltotal"]  # fitness is the negated latency


def test_papers_parallel_unit_example():
    """Sec. 4.1, Symbol-based Analyzer: six scheduling blocks on four parallel units use 0.75 of the peak."""
    hw = w.Device(T_p=1000.0, T_m=100.0, m_l0=1 << 20, m_l1=1 << 20, pu_l1=4, n_l1=32, pu_l2=4, n_l2=1)
    # L2 level: six blocks in the grid, four units
    sg = w.gemm(6, 1, 1, hw=hw)
    _, t64, t32 = oracle.analyze_candidate(sg, [6, 1, 1, 1, 1, 1, 1, 1, 1, 1])
    assert t64["P2c"] == 0.75 and t32["P2c"] == np.float32(0.75)
    # L1 level: six warps (192 threads of 32), four schedulers; no lane is wasted
    sg = w.gemm(192, 1, 1, hw=hw)
    sym, t64, _ = oracle.analyze_candidate(sg, [1, 1, 192, 1, 1, 1, 1, 1, 1, 1])
    assert sym["S4"] == 192 and t64["P1c"] == 0.75 and t64["alpha"] == 1.0
    # both levels at 0.75, everything else at 1 except P0c = 1 + 2/3: U_p = T_p * (5/3) * 0.75 ...
    sg = w.gemm(6 * 192, 1, 1, hw=hw)
    _, t64, _ = oracle.analyze_candidate(sg, [6, 1, 192, 1, 1, 1, 1, 1, 1, 1])
    assert t64["Up"] == pytest.approx(1000.0 * (5.0 / 3.0) * 0.75 * 0.75, rel=1e-15)


def test_capacity_penalties_are_piecewise():
    """P_l0,m = min(m_l0/S1, 1) and P_l1,m = min(m_l1/S3, 1): exactly 1 up to the limit, then the ratio."""
    for m_l0, want in ((14, 1.0), (15, 1.0), (13, 13.0 / 14.0), (7, 0.5)):
        hw = w.Device(T_p=1024.0, T_m=256.0, m_l0=m_l0, m_l1=96, pu_l1=2, n_l1=4, pu_l2=4, n_l2=4)
        _, t64, _ = oracle.analyze_candidate(w.gemm(8, 8, 8, hw=hw), [2, 1, 2, 2, 1, 2, 2, 2, 4, 2])  # S1=14, S3=96
        assert t64["P0m"] == pytest.approx(want, rel=1e-15) and t64["P1m"] == 1.0
    for m_l1, want in ((95, 95.0 / 96.0), (48, 0.5), (97, 1.0)):
        hw = w.Device(T_p=1024.0, T_m=256.0, m_l0=100, m_l1=m_l1, pu_l1=2, n_l1=4, pu_l2=4, n_l2=4)
        _, t64, _ = oracle.analyze_candidate(w.gemm(8, 8, 8, hw=hw), [2, 1, 2, 2, 1, 2, 2, 2, 4, 2])
        assert t64["P1m"] == pytest.approx(want, rel=1e-15) and t64["P0m"] == 1.0


def test_transaction_penalty():
    """P_l2,m = S7 / (ceil(S7/n_l2) * n_l2): 1 on multiples of the transaction length, else the used share."""
    hw = w.Device(T_p=1024.0, T_m=256.0, m_l0=1 << 20, m_l1=1 << 20, pu_l1=1, n_l1=1, pu_l2=1, n_l2=8)
    sg = w.gemm(1, 24, 20, hw=hw)
    # B tile run = B_j, A tile run = D_k
    for bj, dk, want_a, want_b in ((8, 4, 4 / 8, 1.0), (12, 10, 10 / 16, 12 / 16), (24, 20, 20 / 24, 1.0), (3, 5, 5 / 8, 3 / 8)):
        sym, t64, _ = oracle.analyze_candidate(sg, [1, 1, 1, 1, 24 // bj, 1, 1, bj, 20 // dk, dk])
        assert (sym["S7_in0"], sym["S7_in1"], sym["S7_out"]) == (dk, bj, bj)
        assert t64["P2m_in0"] == pytest.approx(want_a, rel=1e-15)
        assert t64["P2m_in1"] == pytest.approx(want_b, rel=1e-15)
        assert t64["P2m_out"] == pytest.approx(want_b, rel=1e-15)


def _gemm_closed_forms(M, N, K, tiles, bytes_=4):
    """Textbook tiling analysis of C[i,j] += A[i,k] B[k,j], vectorised; tiles uint16 [10, n]."""
    t = tiles.astype(np.int64)
    Gi, Vi, Ti, Ii, Gj, Vj, Tj, Ij, Ok, Dk = t
    Bi, Ri, Bj, Rj = Vi * Ti * Ii, Vi * Ii, Vj * Tj * Ij, Vj * Ij
    return {
        "S1": Ri * Rj + Ri + Rj,                      # accumulators + a column of A + a row of B
        "S2": 2 * Ri * Rj,
        "S3": bytes_ * (Bi * Dk + Dk * Bj),
        "S4": Ti * Tj,
        "S6": Gi * Gj,
        "S8": np.full_like(Gi, 2 * M * N * K),
        "S5_in0": bytes_ * M * K * Gj,                # A is re-read once per column of blocks
        "S7_in0": Dk,
        "S5_in1": bytes_ * K * N * Gi,                # B is re-read once per row of blocks
        "S7_in1": Bj,
        "S5_out": np.full_like(Gi, bytes_ * M * N),
        "S7_out": Bj,
    }


def test_brute_force_gemm8_symbols_match_closed_forms():
    """Every schedule of an 8x8x8 GEMM (20*20*4 tilings x 12 annotations): symbols equal the closed forms."""
    sg = w.gemm(8, 8, 8, hw=w.toy_device())
    tiles, ann = w.enumerate_all_schedules(sg)
    assert tiles.shape == (10, 20 * 20 * 4 * 12)
    _, _, sym = oracle.draft_score([sg], [0, tiles.shape[1]], tiles, want_symbols=True)
    want = _gemm_closed_forms(8, 8, 8, tiles)
    for row, name in enumerate(oracle.SYMBOL_NAMES):
        assert np.array_equal(sym[row], want[name]), name


def test_population_symbols_match_closed_forms_large_gemm():
    sg = w.gemm(512, 512, 512)
    tiles, _ = w.sample_population(sg, 20000, seed=3)
    _, _, sym = oracle.draft_score([sg], [0, 20000], tiles, want_symbols=True)
    want = _gemm_closed_forms(512, 512, 512, tiles)
    for row, name in enumerate(oracle.SYMBOL_NAMES):
        assert np.array_equal(sym[row], want[name]), name


def test_flops_do_not_depend_on_tiling_and_traffic_is_monotone():
    """S8 counts the statement's float operations (Sec. 4.1): a property of the subgraph alone.
    S5 of an operand does not grow when the block tile along the axis it is reused over grows."""
    for sg in (w.gemm(512, 512, 512), w.conv2d(1, 64, 56, 56, 64, 3, 3), w.batched_gemm(12, 128, 128, 64),
               w.depthwise_conv2d(1, 512, 28, 28, 3, 3)):
        tiles, _ = w.sample_population(sg, 5000, seed=11)
        _, _, sym = oracle.draft_score([sg], [0, 5000], tiles, want_symbols=True)
        assert np.all(sym[5] == 2 * int(np.prod(sg.extent, dtype=np.int64)))
    sg = w.gemm(512, 512, 512)
    prev_a = None
    for bj in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512):   # grow B_j, all else fixed
        sym, _, _ = oracle.analyze_candidate(sg, [8, 1, 8, 8, 512 // bj, 1, bj, 1, 32, 16])
        assert prev_a is None or sym["S5_in0"] <= prev_a
        assert sym["S5_in1"] == 4 * 512 * 512 * 8
        prev_a = sym["S5_in0"]


def test_penalty_ranges_on_populations():
    """Utilisation factors lie in (0, 1]; P_l0,c = 1 + S2/S1 lies in (1, 3) for a two-operand contraction with q = 1."""
    for sg in (w.gemm(512, 512, 512), w.conv2d(1, 64, 56, 56, 64, 3, 3)):
        tiles, _ = w.sample_population(sg, 300, seed=5)
        for c in range(300):
            _, t64, _ = oracle.analyze_candidate(sg, tiles[:, c])
            for name in ("P0m", "P1m", "P1c", "alpha", "P2c", "P2m_in0", "P2m_in1", "P2m_out"):
                assert 0.0 < t64[name] <= 1.0, name
            assert 1.0 < t64["P0c"] < 3.0
            assert t64["Ltotal"] > 0 and np.isfinite(t64["Ltotal"])


def test_doubling_the_peaks_halves_the_latency_exactly():
    sg1 = w.gemm(512, 512, 512)
    hw2 = w.Device(**{**sg1.hw.__dict__, "T_p": sg1.hw.T_p * 2, "T_m": sg1.hw.T_m * 2})
    sg2 = w.gemm(512, 512, 512, hw=hw2)
    tiles, _ = w.sample_population(sg1, 4096, seed=0)
    a32, a64, _ = oracle.draft_score([sg1], [0, 4096], tiles)
    b32, b64, _ = oracle.draft_score([sg2], [0, 4096], tiles)
    assert np.array_equal(a32, b32 * np.float32(2)) and np.array_equal(a64, b64 * 2)


def test_ablation_flags_reduce_to_the_plain_roofline_sum():
    """Without both penalty families (Table 10 switches) Eq. 1 is flops/T_p + bytes/T_m with closed-form GEMM traffic."""
    sg = w.gemm(512, 512, 512)
    tiles, _ = w.sample_population(sg, 4096, seed=9)
    cf = _gemm_closed_forms(512, 512, 512, tiles)
    T_p, T_m = float(np.float32(sg.hw.T_p)), float(np.float32(sg.hw.T_m))
    want = cf["S8"] / T_p + (cf["S5_in0"] + cf["S5_in1"] + cf["S5_out"]) / T_m
    _, s64, _ = oracle.draft_score([sg], [0, 4096], tiles, flags=oracle.NO_COMPUTE_PENALTY | oracle.NO_MEMORY_PENALTY)
    assert np.allclose(-s64, want, rtol=1e-14, atol=0)
    # each switch alone touches only its own family
    for c in range(20):
        _, full, _ = oracle.analyze_candidate(sg, tiles[:, c])
        _, noc, _ = oracle.analyze_candidate(sg, tiles[:, c], flags=oracle.NO_COMPUTE_PENALTY)
        _, nom, _ = oracle.analyze_candidate(sg, tiles[:, c], flags=oracle.NO_MEMORY_PENALTY)
        assert noc["Up"] == T_p and noc["Um_in0"] == full["Um_in0"]
        assert nom["Um_in0"] == T_m and nom["Up"] == full["Up"]


def test_unit_conv_equals_gemm_and_batch_one_equals_gemm():
    """A 1x1 convolution over a 1xW image row is the GEMM [K x W x C]; a batch of one is the plain GEMM.

    The weight tensor [k,c,1,1] has an innermost dimension of length 1, so its S7 is 1 where the GEMM
    operand [k,c] has D_c; with a transaction length of one element that does not reach the score.
    """
    hw = w.Device(T_p=1024.0, T_m=256.0, m_l0=8, m_l1=64, pu_l1=2, n_l1=4, pu_l2=4, n_l2=1)
    g = w.gemm(16, 24, 32, hw=hw)                                   # C[k, w] += Wt[k, c] * I[c, w]
    cv = w.conv2d(1, 32, 1, 24, 16, 1, 1, stride=1, pad=0, hw=hw)   # axes n,k,h,w | c,r,s
    bg = w.batched_gemm(1, 16, 24, 32, hw=hw)
    tiles, _ = w.sample_population(g, 2000, seed=2)
    ones4, ones2 = np.ones((4, 2000), np.uint16), np.ones((2, 2000), np.uint16)
    # conv slots: n(4) k(4) h(4) w(4) c(2) r(2) s(2); gemm i->k, j->w, k->c
    ctiles = np.vstack([ones4, tiles[0:4], ones4, tiles[4:8], tiles[8:10], ones2, ones2])
    btiles = np.vstack([ones4, tiles])
    g32, g64, gs = oracle.draft_score([g], [0, 2000], tiles, want_symbols=True)
    c32, c64, cs = oracle.draft_score([cv], [0, 2000], ctiles, want_symbols=True)
    b32, b64, bs = oracle.draft_score([bg], [0, 2000], btiles, want_symbols=True)
    assert np.array_equal(g32, b32) and np.array_equal(g64, b64) and np.array_equal(gs, bs)
    # in the conv the image is input 0 and the weights input 1: the two operands swap places
    swap = [0, 1, 2, 3, 4, 5, 8, 9, 6, 7, 10, 11]
    keep = [r for r in range(12) if r != 9]
    assert np.array_equal(gs[swap][keep], cs[keep]) and np.all(cs[9] == 1)
    assert np.allclose(g64, c64, rtol=1e-15, atol=0)


def test_conv_halo_footprint_closed_form():
    """Block tile of the image is (B_h-1)*stride + D_r by (B_w-1)*stride + D_s per channel; borders ignored."""
    for stride in (1, 2):
        sg = w.conv2d(1, 8, 17 if stride == 2 else 8, 17 if stride == 2 else 8, 4, 3, 3, stride=stride, pad=1, hw=w.toy_device())
        tiles, _ = w.sample_population(sg, 3000, seed=4)
        t = tiles.astype(np.int64)
        B = [t[4 * a + 1] * t[4 * a + 2] * t[4 * a + 3] for a in range(4)]
        G = np.prod(t[[0, 4, 8, 12]], axis=0)
        O = t[16] * t[18] * t[20]
        Dc, Dr, Ds = t[17], t[19], t[21]
        img = B[0] * Dc * ((B[2] - 1) * stride + Dr) * ((B[3] - 1) * stride + Ds)
        wgt = B[1] * Dc * Dr * Ds
        _, _, sym = oracle.draft_score([sg], [0, 3000], tiles, want_symbols=True)
        assert np.array_equal(sym[2], 4 * (img + wgt))
        assert np.array_equal(sym[6], 4 * G * O * img) and np.array_equal(sym[8], 4 * G * O * wgt)
        assert np.array_equal(sym[7], (B[3] - 1) * stride + Ds) and np.array_equal(sym[9], Ds)


def test_binary32_path_tracks_binary64_within_1e5_on_all_workload_shapes():
    cases = [w.make_config(0), w.make_config(1, scale=0.25), w.make_config(2, scale=0.05), w.make_config(4, scale=0.002)]
    for wl in cases:
        s32, s64, _ = oracle.draft_score(wl.subgraphs, wl.seg_off, wl.tiles)
        rel = np.abs(s32.astype(np.float64) - s64) / np.abs(s64)
        assert rel.max() <= 1e-5, (wl.name, rel.max())
        assert np.all(s64 < 0) and np.all(np.isfinite(s32))


def test_int64_symbols_round_to_nearest_even_when_converted():
    """A traffic count above 2^24 that binary32 cannot hold: the binary32 path must see its nearest-even rounding."""
    hw = w.Device(T_p=1.0, T_m=1.0, m_l0=1 << 30, m_l1=1 << 30, pu_l1=1, n_l1=1, pu_l2=1, n_l2=1)
    sg = w.gemm(4099, 4097, 3, hw=hw)
    sym, t64, t32 = oracle.analyze_candidate(sg, [4099, 1, 1, 1, 4097, 1, 1, 1, 3, 1], flags=oracle.NO_COMPUTE_PENALTY | oracle.NO_MEMORY_PENALTY)
    s5 = sym["S5_in0"]
    assert s5 == 4 * 4099 * 3 * 4097 and s5 > (1 << 24) and int(np.float32(s5)) != s5
    assert t32["Lm_in0"] == np.float32(s5) and t64["Lm_in0"] == float(s5)


def test_bad_factors_are_rejected():
    sg = w.gemm(8, 8, 8, hw=w.toy_device())
    with pytest.raises(oracle.OracleError):
        oracle.analyze_candidate(sg, [2, 1, 2, 2, 1, 2, 2, 2, 4, 4])     # k factors multiply to 16
    with pytest.raises(oracle.OracleError):
        oracle.analyze_candidate(sg, [0, 1, 2, 2, 1, 2, 2, 2, 4, 2])
