"""Parity of the HIP library with the CPU oracle, through the C boundary, on the same seeded inputs.

Bars: integer symbols and top-k index lists bit-exact; draft scores within 1e-5 relative of the oracle's binary64
value in the default (fused) arithmetic -- the test asserts the tighter 2e-6 that its error analysis gives -- and
bit-exact against the oracle's binary32 path under PRUNER_REFERENCE_ROUNDING; verify scores within 2e-2 relative and
never below 2^-9 of the summed size of the last layer's terms, per candidate (oracle.verify_tolerance; its footing is
shown on the CPU in tests/test_oracle_verify.py).  Selection is compared on one and
the same score array (the library's), and end to end against the oracle under reference rounding.
"""
import numpy as np
import pytest

import oracle
import workloads as w

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2402_02361_amd as P
    P.load_library()
    return P


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


FUSED_TOL = 2e-6     # about a dozen binary32 roundings and one 1-ulp reciprocal per statement group, all terms positive


def check_draft(P, subgraphs, seg_off, tiles, flags=0, pitch_pad=0, symbols=True):
    n = int(seg_off[-1])
    if pitch_pad:
        tiles = np.concatenate([tiles, np.ones((tiles.shape[0], pitch_pad), np.uint16)], axis=1)
    o32, o64, osym = oracle.draft_score(subgraphs, seg_off, tiles, flags=flags, want_symbols=symbols)
    dt = dev(tiles)
    result = None
    bits = {}
    for mode in (P.REFERENCE_ROUNDING, P.FUSED_ARITHMETIC, 0):
        out = P.draft_score(subgraphs, seg_off, dt, flags=flags | mode, symbols=symbols)
        torch.cuda.synchronize()
        g32, gsym = out if symbols else (out, None)
        g32 = g32.cpu().numpy()
        if symbols:
            gsym = gsym.cpu().numpy()
            for r, name in enumerate(oracle.SYMBOL_NAMES):
                bad = np.flatnonzero(gsym[r] != osym[r])
                assert bad.size == 0, (mode, name, bad[:5], gsym[r][bad[:5]], osym[r][bad[:5]])
            # the launch without the symbol dump is a different kernel instance (it may form products in binary32)
            plain = P.draft_score(subgraphs, seg_off, dt, flags=flags | mode).cpu().numpy()
            bad = np.flatnonzero(plain.view(np.uint32) != g32.view(np.uint32))
            assert bad.size == 0, (mode, "no-dump kernel", bad[:5], plain[bad[:5]], g32[bad[:5]])
        bits[mode] = g32.view(np.uint32)
        if mode == P.REFERENCE_ROUNDING:
            bad = np.flatnonzero(g32.view(np.uint32) != o32.view(np.uint32))
            assert bad.size == 0, (bad[:5], g32[bad[:5]], o32[bad[:5]])
            result = g32
        rel = np.abs(g32.astype(np.float64) - o64) / np.abs(o64)
        assert n == 0 or rel.max() <= (1e-5 if mode == P.REFERENCE_ROUNDING else FUSED_TOL), (mode, rel.max(), int(rel.argmax()))
    # without a switch: the oracle's bits from a call that runs as one launch; the fused form in the per-class launches,
    # which populations of 2^20 candidates and more get when every segment start and the pitch allow 8-byte loads
    per_class = n >= (1 << 20) and tiles.shape[1] % 4 == 0 and all(int(o) % 4 == 0 for o in list(seg_off)[:-1])
    assert np.array_equal(bits[0], bits[P.FUSED_ARITHMETIC] if per_class else bits[P.REFERENCE_ROUNDING]), per_class
    return result


# ---- draft model ---------------------------------------------------------------------------------------------------

def test_draft_worked_example_bits(P):
    """The hand-computed 8x8x8 example: L_total = 1799/120, binary32 0x416FDDDD, score is its negation."""
    sg = w.gemm(8, 8, 8, hw=w.toy_device())
    tiles = np.array([2, 1, 2, 2, 1, 2, 2, 2, 4, 2], np.uint16)[:, None]
    g = check_draft(P, [sg], [0, 1], tiles)
    assert g.view(np.uint32)[0] == 0xC16FDDDD


def test_draft_config0_full(P):
    wl = w.make_config(0)
    check_draft(P, wl.subgraphs, wl.seg_off, wl.tiles)


def test_draft_config1_full(P):
    wl = w.make_config(1)
    check_draft(P, wl.subgraphs, wl.seg_off, wl.tiles)


def test_draft_config2_full(P):
    wl = w.make_config(2)
    check_draft(P, wl.subgraphs, wl.seg_off, wl.tiles)


def test_draft_config4_scaled(P):
    wl = w.make_config(4, scale=1 / 64)     # 262,144 + 65,536 candidates, fragment mode + depthwise conv
    check_draft(P, wl.subgraphs, wl.seg_off, wl.tiles)


def test_draft_every_schedule_of_a_tiny_gemm(P):
    sg = w.gemm(8, 8, 8, hw=w.toy_device())
    tiles, _ = w.enumerate_all_schedules(sg)
    check_draft(P, [sg], [0, tiles.shape[1]], tiles)


@pytest.mark.parametrize("offs", [[0, 1, 2, 1003, 1003, 5001], [0, 2, 1002, 4098], [0, 4, 1028, 5000]])
def test_draft_ragged_segments_and_alignment(P, offs):
    """Odd segment starts force the 1- and 2-wide load paths; an empty segment and a 1-candidate segment ride along."""
    sgs = [w.gemm(512, 512, 512), w.batched_gemm(12, 128, 128, 64), w.conv2d(1, 64, 56, 56, 64, 3, 3),
           w.depthwise_conv2d(1, 512, 28, 28, 3, 3), w.gemm(128, 768, 3072)][: len(offs) - 1]
    seg = np.array(offs, np.int64)
    slots = max(w.n_slots(s) for s in sgs)
    tiles = np.zeros((slots, int(seg[-1])), np.uint16)
    for t, sg in enumerate(sgs):
        cnt = int(seg[t + 1] - seg[t])
        if cnt:
            tl, _ = w.sample_population(sg, cnt, seed=21, stream=t)
            tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
    check_draft(P, sgs, seg, tiles)
    check_draft(P, sgs, seg, tiles, pitch_pad=3)
    # a candidate's score does not depend on the load width its call runs at: the fused form too gives the same bits
    # from a pitch that allows the wide loads and from one that forces single loads
    padded = np.concatenate([tiles, np.ones((tiles.shape[0], 3), np.uint16)], axis=1)
    a = P.draft_score(sgs, seg, dev(tiles), flags=P.FUSED_ARITHMETIC).cpu().numpy()
    b = P.draft_score(sgs, seg, dev(padded), flags=P.FUSED_ARITHMETIC).cpu().numpy()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_draft_generic_nest_and_odd_divisors(P):
    """Access patterns outside the built-in classes (B stored transposed, a strided 1-d correlation with one input
    dimension of two terms), hardware constants that are not powers of two, and a single-input statement."""
    hw = w.Device(T_p=3.3e12, T_m=4.1e11, m_l0=96, m_l1=20000, pu_l1=3, n_l1=24, pu_l2=7, n_l2=5)
    d = lambda *t: tuple(t)
    bt = w.Subgraph("gemm_bt", 2, 1, (96, 80, 72), 4, 3, 4, (0, 0, 0),
                    (w.Buffer((d((0, 1)), d((2, 1)))), w.Buffer((d((1, 1)), d((2, 1))))), w.Buffer((d((0, 1)), d((1, 1)))), hw)
    corr = w.Subgraph("corr1d", 1, 1, (120, 9), 4, 2, 2, (0, 0, 0),
                      (w.Buffer((d((0, 3), (1, 2)),)), w.Buffer((d((1, 1)),))), w.Buffer((d((0, 1)),)), hw)
    rsum = w.Subgraph("rowsum", 1, 1, (60, 84), 4, 2, 4, (0, 0, 0), (w.Buffer((d((0, 1)), d((1, 1)))),), w.Buffer((d((0, 1)),)), hw)
    for sg in (bt, corr, rsum):
        tiles, _ = w.sample_population(sg, 3001, seed=6)
        check_draft(P, [sg], [0, 3001], tiles)
    for pu in (1, 80, 108, 304):
        sg = w.gemm(512, 512, 512, hw=w.Device(**{**w.a100_like(4).__dict__, "pu_l2": pu, "pu_l1": 1 + pu % 5}))
        tiles, _ = w.sample_population(sg, 4096, seed=pu)
        check_draft(P, [sg], [0, 4096], tiles)


def test_draft_one_launch_per_class(P):
    """Above 2^20 candidates the library launches one kernel per loop-nest class: all five classes, interleaved in
    the segment order, one class twice, with segment lengths that leave partial chunks."""
    hw = w.Device(T_p=3.3e12, T_m=4.1e11, m_l0=96, m_l1=20000, pu_l1=3, n_l1=24, pu_l2=7, n_l2=5)
    d = lambda *t: tuple(t)
    bt = w.Subgraph("gemm_bt", 2, 1, (96, 80, 72), 4, 3, 4, (0, 0, 0),
                    (w.Buffer((d((0, 1)), d((2, 1)))), w.Buffer((d((1, 1)), d((2, 1))))), w.Buffer((d((0, 1)), d((1, 1)))), hw)
    sgs = [w.conv2d(1, 64, 56, 56, 64, 3, 3), w.gemm(512, 512, 512), bt, w.depthwise_conv2d(1, 512, 28, 28, 3, 3),
           w.batched_gemm(12, 128, 128, 64), w.gemm(128, 768, 3072)]
    lens = [200004, 150000, 180004, 250000, 170008, 150004]             # every offset and the pitch stay multiples of 4
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    assert seg[-1] >= 1 << 20
    slots = max(w.n_slots(s) for s in sgs)
    tiles = np.zeros((slots, int(seg[-1])), np.uint16)
    for t, sg in enumerate(sgs):
        tl, _ = w.sample_population(sg, lens[t], seed=33, stream=t)
        tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
    check_draft(P, sgs, seg, tiles)


@pytest.mark.parametrize("lens,flags", [([1285900, 290336, 43992], 1), ([1135293], 2), ([1285516, 270448, 249705], 0)])
def test_draft_scores_do_not_depend_on_the_launch_shape(P, lens, flags):
    """A large segment beside small ones, and ends that are not multiples of four behind aligned starts: the same
    candidates are scored by the per-class launches and, for the symbol dump, by the single launch, whose workgroups
    cover different numbers of candidates (some tabulate P_l2,m, some do not).  check_draft asserts equal bits between
    the two in every arithmetic mode."""
    sgs = [w.gemm(8, 3072, 1000), w.gemm(1024, 256, 256), w.batched_gemm(2, 100, 128, 1000)][: len(lens)]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    slots = max(w.n_slots(s) for s in sgs)
    tiles = np.zeros((slots, int(seg[-1])), np.uint16)
    for t, sg in enumerate(sgs):
        tl, _ = w.sample_population(sg, lens[t], seed=10, stream=t)
        tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
    check_draft(P, sgs, seg, tiles, flags=flags, pitch_pad=(-int(seg[-1])) % 4)


def test_draft_fragment_mode_unaligned_tiles(P):
    """Inner tiles that are not whole fragments: the fragment-utilisation factor drops below one."""
    hw = w.Device(T_p=1024.0, T_m=256.0, m_l0=1024, m_l1=8192, pu_l1=2, n_l1=4, pu_l2=4, n_l2=4)
    sg = w.gemm(48, 64, 64, dtype_bytes=2, hw=hw, rd_levels=3, frag=(16, 16, 16))
    free = w.gemm(48, 64, 64, dtype_bytes=2, hw=hw, rd_levels=3)          # same nest, unconstrained factorisations
    tiles, _ = w.sample_population(free, 5000, seed=12)
    g = check_draft(P, [sg], [0, 5000], tiles)
    ex = np.array([1, 2, 1, 24, 2, 1, 2, 16, 2, 2, 16], np.uint16)[:, None]
    g = check_draft(P, [sg], [0, 1], ex)
    assert g[0] == np.float32(-(104 + 7168 / 391))                       # hand-computed: tests/golden, gemm48_fragment_unaligned


def test_draft_ablation_flags(P):
    wl = w.make_config(0)
    for flags in (1, 2, 3):
        check_draft(P, wl.subgraphs, wl.seg_off, wl.tiles, flags=flags)


def test_draft_is_deterministic_and_ignores_unused_slots(P):
    wl = w.make_config(2, scale=0.1)
    t = dev(wl.tiles)
    a = P.draft_score(wl.subgraphs, wl.seg_off, t).cpu().numpy()
    junk = wl.tiles.copy()
    lo, hi = wl.seg_off[0], wl.seg_off[1]
    junk[10:, lo:hi] = 7                                                   # slots the 10-slot GEMM does not own
    b = P.draft_score(wl.subgraphs, wl.seg_off, dev(junk)).cpu().numpy()
    c = P.draft_score(wl.subgraphs, wl.seg_off, t).cpu().numpy()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32)) and np.array_equal(a.view(np.uint32), c.view(np.uint32))


# ---- selection -------------------------------------------------------------------------------------------------------

def check_topk(P, score, seg_off, k):
    oi, ov = oracle.topk(score, seg_off, k)
    gi, gv = P.topk(dev(score), seg_off, k)
    torch.cuda.synchronize()
    gi, gv = gi.cpu().numpy(), gv.cpu().numpy()
    bad = np.argwhere(gi != oi)
    assert bad.size == 0, (bad[:5], gi[tuple(bad[0])], oi[tuple(bad[0])])
    assert np.array_equal(gv.view(np.uint32), ov.view(np.uint32))


@pytest.mark.parametrize("k", [1, 7, 64, 512, 4096])
def test_topk_small_route_with_ties(P, k):
    rng = np.random.default_rng(k)
    seg = np.array([0, 5000, 9096, 39000, 39000 + 4096], np.int64)                 # (the longest stays within one workgroup's limit)
    score = rng.integers(-300, 300, size=int(seg[-1])).astype(np.float32) / 8      # few distinct values: many exact ties
    check_topk(P, score, seg, k)
    check_topk(P, rng.normal(size=int(seg[-1])).astype(np.float32), seg, k)


@pytest.mark.parametrize("k", [1, 2, 31, 32, 63, 64])
def test_topk_tiny_route(P, k):
    """Segments of at most 8192 entries with k up to 64 (the final selection's shape): four wavefronts per segment, keys in
    registers.  Ragged lengths down to k itself, full-length segments, few distinct values (the tie cut by index runs),
    all-equal segments (ties only), signed zeros and infinities among the best."""
    rng = np.random.default_rng(500 + k)
    lens = [k, k + 1, 64, 65, 255, 256, 257, 1000, 4096, 8191, 8192, 512, 8192]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n = int(seg[-1])
    check_topk(P, rng.normal(size=n).astype(np.float32), seg, k)
    check_topk(P, rng.integers(-3, 3, size=n).astype(np.float32), seg, k)          # six values: far more ties than k
    check_topk(P, (rng.integers(-40, 40, size=n) / 4).astype(np.float32), seg, k)   # entries above T and ties together
    check_topk(P, np.zeros(n, np.float32), seg, k)
    special = rng.normal(size=n).astype(np.float32)
    special[rng.integers(0, n, n // 50)] = np.inf
    special[rng.integers(0, n, n // 50)] = -np.inf
    special[rng.integers(0, n, n // 3)] = 0.0
    special[rng.integers(0, n, n // 3)] = -0.0
    check_topk(P, special, seg, k)
    check_topk(P, -np.abs(special), seg, k)                                          # zeros of both signs are the best: ties by index
    many = np.concatenate([[0], np.cumsum(np.full(300, 70))]).astype(np.int64)       # more segments than travel as arguments
    check_topk(P, rng.normal(size=int(many[-1])).astype(np.float32), many, min(k, 64))


def test_topk_special_values(P):
    score = np.array([0.0, -0.0, np.inf, -np.inf, 1.0, -0.0, 0.0, -1.0] * 3, np.float32)
    check_topk(P, score, [0, 8, 24], 8)
    check_topk(P, score, [0, 24], 24)
    check_topk(P, np.zeros(20000, np.float32), [0, 20000], 100)                    # every entry ties
    check_topk(P, np.full(5000, -np.inf, np.float32), [0, 5000], 5000 - 904)
    tiny = np.array([1e-45, -1e-45, 3e-39, 1e-38, -3e-39, 0.0], np.float32)         # denormals order like any value
    check_topk(P, tiny, [0, 6], 6)


@pytest.mark.parametrize("k", [1, 32, 4096])
def test_topk_large_route(P, k):
    rng = np.random.default_rng(100 + k)
    seg = np.array([0, 300001, 300001 + 4096, 700000], np.int64)                    # one segment above the one-workgroup limit
    n = int(seg[-1])
    check_topk(P, rng.normal(size=n).astype(np.float32) - 5, seg, k)
    check_topk(P, rng.integers(-50, 50, size=n).astype(np.float32), seg, k)         # about 7,000 entries per value
    check_topk(P, rng.integers(-20, 20, size=n).astype(np.float32), seg, k)         # the tie quota spans several overflowed lists
    check_topk(P, rng.integers(-150, 150, size=n).astype(np.float32), seg, k)       # entries above T and ties together
    check_topk(P, np.zeros(n, np.float32), seg, k)                                  # ties only: pure index order


def test_topk_large_route_many_segments_and_dense_ties(P):
    """Eight long segments with k = 4096 (the ranking of a segment is shared out over 128 workgroups), and the
    explorer loop's kind of scores: the best value shared by two per cent of a long segment, so that the k best are
    ties only and the tie quota runs over a dozen spans whose tie lists overflow."""
    rng = np.random.default_rng(77)
    n = 8 * 150000
    seg = np.arange(9, dtype=np.int64) * 150000
    check_topk(P, rng.normal(size=n).astype(np.float32), seg, 4096)
    check_topk(P, np.round(rng.normal(size=n) * 40).astype(np.float32), seg, 4096)       # entries above T and ties in every segment
    m = 1 << 21
    clipped = np.minimum(rng.normal(size=m), 2.0).astype(np.float32)
    check_topk(P, clipped, [0, m], 4096)
    check_topk(P, clipped, [0, m // 2, m], 4096)
    check_topk(P, clipped, [0, m], 100)


@pytest.mark.parametrize("k", [1, 100, 1000])
def test_topk_sparse_selection_steps_over_blocks(P, k):
    """At most one entry in 1024 of the longest segment selected: the pass that sets entries aside reads only the blocks of
    256 entries whose largest key reaches the rank-k bucket.  Segment starts that are multiples of 4 but not of 256; the best
    entries crowded into a few blocks, spread one per block, and sitting in a block's first and last place; ties with the
    k-th value that run across block and span boundaries; infinities; a segment of equal values (every block is needed: the
    workgroups fall back to plain sweeps); the last block of a segment short of 256 entries."""
    rng = np.random.default_rng(500 + k)
    seg = np.array([0, 1200004, 1200004 + 1100000 + 36, 3500000 - 3], np.int64)
    n = int(seg[-1])
    base = (-np.exp(rng.normal(size=n))).astype(np.float32)
    check_topk(P, base, seg, k)
    crowded = base.copy()
    for s in range(3):
        at = int(seg[s]) + 256 * 1000 + np.arange(2 * k)            # 2k neighbours, the best of their segment
        crowded[at] = -1e-6 * (1 + rng.integers(0, 50, size=2 * k)).astype(np.float32)   # few distinct values: ties at the cut
    check_topk(P, crowded, seg, k)
    edges = base.copy()
    for s in range(3):
        first = int(seg[s]) + 256 * np.arange(k, dtype=np.int64) * 3   # a block's first entry (blocks count from the segment's begin)
        edges[first] = np.float32(-1e-7)
        edges[first[: k // 2 + 1] + 255] = np.float32(-1e-7)           # and its last: all tie, the lowest indices win
    edges[int(seg[1]) - 1] = np.inf                                     # the last entry of a segment, in its short last block
    edges[int(seg[1])] = np.inf
    check_topk(P, edges, seg, k)
    check_topk(P, np.full(n, -2.5, np.float32), seg, k)
    two = np.where(rng.random(n) < 0.5, np.float32(-1.0), np.float32(-3.0)).astype(np.float32)
    check_topk(P, two, seg, k)


def test_topk_on_draft_scores_of_each_config(P):
    for idx, scale in ((0, 1.0), (1, 1.0), (2, 1.0), (4, 1 / 16)):
        wl = w.make_config(idx, scale=scale)
        s32, _, _ = oracle.draft_score(wl.subgraphs, wl.seg_off, wl.tiles)
        check_topk(P, s32, wl.seg_off, wl.k_draft)


# ---- verify model ------------------------------------------------------------------------------------------------------

def gpu_weights(m):
    return {k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in m.items()}


def check_verify(P, feat, n_stmt, m):
    o32, o64, mag = oracle.verify(feat, n_stmt, m, want_mag=True)
    g = P.verify_score(dev(feat), dev(np.asarray(n_stmt, np.int32)), gpu_weights(m))
    torch.cuda.synchronize()
    g = g.cpu().numpy()
    tol = oracle.verify_tolerance(o32, mag)      # 2e-2 relative, at least 2^-9 of the summed term sizes, per candidate
    bad = np.flatnonzero(~(np.abs(g - o32) <= tol))
    assert bad.size == 0, (bad[:5], g[bad[:5]], o32[bad[:5]])
    return g, o32


def test_verify_hand_sized_values_through_zero_padding(P):
    """Weights that are zero outside a 2x2 corner turn the 164-256-256-1 network into the hand-computed 2-2-2-1 one."""
    bf = w.f32_to_bf16_bits
    W1 = np.zeros((256, 164), np.float32); W1[:2, :2] = [[1, -1], [2, 0]]
    W2 = np.zeros((256, 256), np.float32); W2[:2, :2] = [[1, 1], [-1, 2]]
    w3 = np.zeros(256, np.float32); w3[:2] = [2, -1]
    b1 = np.zeros(256, np.float32); b1[:2] = [0, -3]
    b2 = np.zeros(256, np.float32); b2[:2] = [1, 0]
    m = {"W1": bf(W1), "b1": b1, "W2": bf(W2), "b2": b2, "w3": bf(w3), "b3": 0.5}
    feat = np.zeros((2, 8, 164), np.float32)
    feat[0, 0, :2], feat[0, 1, :2], feat[1, 0, :2], feat[1, 1, :2] = (3, 1), (1, 5), (2, 2), (9, 9)
    g, o = check_verify(P, feat, [2, 1], m)
    assert list(g) == [11.0, 2.5] and list(o) == [11.0, 2.5]


def test_verify_random_weights_ragged_statements(P):
    m = w.make_mlp_weights(seed=1)
    rng = np.random.default_rng(3)
    for n_d in (1, 7, 8, 9, 333, 2048 + 5):
        n_stmt = rng.integers(0, 9, size=n_d).astype(np.int32)
        feat = w.make_statement_features(np.arange(n_d) * 31 + 5, n_stmt, pad_value=1e6)   # garbage in padded rows
        check_verify(P, feat, n_stmt, m)


def test_verify_beyond_the_in_kernel_row_numbering(P):
    """17,001 candidates (66 per workgroup, in groups of eight), few rows each, with a run of full candidates so that tiles do
    split candidates and the carried partial sums are used."""
    m = w.make_mlp_weights(seed=1)
    rng = np.random.default_rng(9)
    n_d = 17001
    n_stmt = rng.integers(0, 3, size=n_d).astype(np.int32)
    n_stmt[100:140] = 8                                   # a run of full candidates, so that tiles do split some
    feat = w.make_statement_features(np.arange(n_d) * 7 + 1, n_stmt, pad_value=-3e5)
    check_verify(P, feat, n_stmt, m)


def test_verify_set_larger_than_one_launch_takes(P):
    """600,001 candidates: more than 2048 per compute unit, so the call is cut into two launches.  Nearly all candidates
    have no statement (their features are never read); a sample with statements, among them the candidates on both sides
    of the cut and the last one, is checked against the oracle, and everybody else must score 0."""
    m = w.make_mlp_weights(seed=1)
    rng = np.random.default_rng(12)
    n_d = 600001
    cut = 2048 * torch.cuda.get_device_properties(0).multi_processor_count
    pick = np.unique(np.concatenate([rng.integers(0, n_d, 1500), np.arange(cut - 20, min(cut + 20, n_d)), [0, n_d - 1]]))
    pick = pick[pick < n_d]
    n_stmt = np.zeros(n_d, np.int32)
    n_stmt[pick] = rng.integers(1, 9, size=len(pick))
    rows = w.make_statement_features(pick * 3 + 1, n_stmt[pick], pad_value=4e4)
    feat = torch.full((n_d, 8, 164), float("nan"), dtype=torch.float32, device="cuda")     # never read where n_stmt is 0
    feat[torch.from_numpy(pick).cuda()] = dev(rows)
    got = P.verify_score(feat, dev(n_stmt), gpu_weights(m)).cpu().numpy()
    want, _, mag = oracle.verify(rows, n_stmt[pick], m, want_mag=True)
    assert np.all(np.abs(got[pick] - want) <= oracle.verify_tolerance(want, mag))
    rest = np.ones(n_d, bool)
    rest[pick] = False
    assert not got[rest].any()


def test_verify_in_kernel_row_numbering_at_its_limits(P):
    """16383 candidates, mostly without rows, and counts outside 0..8."""
    m = w.make_mlp_weights(seed=1)
    rng = np.random.default_rng(10)
    n_d = 16383
    n_stmt = (rng.random(n_d) < 0.08).astype(np.int32) * rng.integers(1, 9, size=n_d).astype(np.int32)
    feat = w.make_statement_features(np.arange(n_d) * 3 + 2, n_stmt, pad_value=7e4)
    check_verify(P, feat, n_stmt, m)
    wild = n_stmt.copy()
    wild[::5] = np.where(wild[::5] == 0, -4, wild[::5])   # negative counts read as 0 ...
    g, _ = check_verify(P, feat, np.clip(wild, 0, 8), m)
    g2 = P.verify_score(dev(feat), dev(wild), gpu_weights(m)).cpu().numpy()
    assert np.array_equal(g, g2)


def test_verify_in_kernel_row_numbering_with_every_row_valid(P):
    """16383 candidates of 8 statements each (every tile full, no candidate split: 8 divides 64); a sample of candidates
    against the oracle (a candidate's score depends on its own rows only)."""
    m = w.make_mlp_weights(seed=1)
    n_d = 16383
    n_stmt = np.full(n_d, 8, np.int32)
    feat = w.make_statement_features(np.arange(n_d) * 5 + 3, n_stmt)
    got = P.verify_score(dev(feat), dev(n_stmt), gpu_weights(m)).cpu().numpy()
    pick = np.unique(np.concatenate([np.arange(0, 40), np.arange(n_d - 40, n_d), np.random.default_rng(4).integers(0, n_d, 300)]))
    want, _, mag = oracle.verify(feat[pick], n_stmt[pick], m, want_mag=True)
    assert np.all(np.abs(got[pick] - want) <= oracle.verify_tolerance(want, mag))
    assert np.isfinite(got).all()


def test_verify_zero_weights_and_all_padding(P):
    m = w.make_mlp_weights(seed=1)
    z = {k: (np.zeros_like(v) if isinstance(v, np.ndarray) else 0.375) for k, v in m.items()}
    n_stmt = np.array([0, 1, 3, 8, 5, 0], np.int32)
    feat = w.make_statement_features(np.arange(6), n_stmt)
    g, _ = check_verify(P, feat, n_stmt, z)
    assert np.array_equal(g, (n_stmt * 0.375).astype(np.float32))
    g, _ = check_verify(P, feat, np.zeros(6, np.int32), m)
    assert np.all(g == 0)


# ---- draft + selection in one call ------------------------------------------------------------------------------------

def check_prior_filter(P, subgraphs, seg_off, tiles, k, flags=0):
    """pruner_prior_filter against the two separate calls (bit for bit) and, under reference rounding, the oracle."""
    dt = dev(tiles)
    score, idx, val = P.prior_filter(subgraphs, seg_off, dt, k, flags=flags)
    s2 = P.draft_score(subgraphs, seg_off, dt, flags=flags)
    i2, v2 = P.topk(s2, seg_off, k)
    torch.cuda.synchronize()
    score, idx, val = score.cpu().numpy(), idx.cpu().numpy(), val.cpu().numpy()
    assert np.array_equal(score.view(np.uint32), s2.cpu().numpy().view(np.uint32))
    assert np.array_equal(idx, i2.cpu().numpy()) and np.array_equal(val.view(np.uint32), v2.cpu().numpy().view(np.uint32))
    if flags & P.REFERENCE_ROUNDING:
        o32, _, _ = oracle.draft_score(subgraphs, seg_off, tiles, flags=flags & 3)
        oi, ov = oracle.topk(o32, seg_off, k)
        assert np.array_equal(score.view(np.uint32), o32.view(np.uint32))
        assert np.array_equal(idx, oi) and np.array_equal(val.view(np.uint32), ov.view(np.uint32))
    else:
        oi, ov = oracle.topk(score, seg_off, k)
        assert np.array_equal(idx, oi) and np.array_equal(val.view(np.uint32), ov.view(np.uint32))


@pytest.mark.parametrize("flags", [0, 4, 8])
def test_prior_filter_large_route_counts_digits_in_the_draft_kernel(P, flags):
    wl = w.make_config(4, scale=1 / 8)                    # 2M + 512K candidates: per-class launches, large selection route
    check_prior_filter(P, wl.subgraphs, wl.seg_off, wl.tiles, wl.k_draft, flags)
    wl = w.make_config(2)                                 # 1,000,000 in 20 segments: single launch, small route
    check_prior_filter(P, wl.subgraphs, wl.seg_off, wl.tiles, wl.k_draft, flags)


def test_prior_filter_odd_alignment_and_mixed_classes(P):
    """Segment starts that force the narrow load widths (no digit counting in the draft kernel) with one segment
    long enough for the large selection route; then the aligned case with four loop-nest classes."""
    sgs = [w.gemm(512, 512, 512), w.batched_gemm(12, 128, 128, 64), w.conv2d(1, 64, 56, 56, 64, 3, 3), w.depthwise_conv2d(1, 512, 28, 28, 3, 3)]
    for lens in ([150001, 70001, 3001, 40002], [150000, 70004, 3000, 40004]):
        seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        slots = max(w.n_slots(s) for s in sgs)
        tiles = np.zeros((slots, int(seg[-1])), np.uint16)
        for t, sg in enumerate(sgs):
            tl, _ = w.sample_population(sg, lens[t], seed=44, stream=t)
            tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
        check_prior_filter(P, sgs, seg, tiles, 512)
        check_prior_filter(P, sgs, seg, tiles, 512, flags=4)
        check_prior_filter(P, sgs, seg, tiles, 512, flags=8)


@pytest.mark.parametrize("k", [1, 33, 64])
def test_prior_filter_short_segments(P, k):
    """Segments of at most 8192 candidates with k at most 64 (the selection's route for short segments) behind the draft
    kernel in one call.  Four loop-nest classes, lengths from k itself to 8192, aligned starts and odd ones (narrow load
    widths), the three arithmetic modes and the ablation switches; then one segment of 8193 and k = 65 (the next route)."""
    sgs = [w.gemm(512, 512, 512), w.batched_gemm(12, 128, 128, 64), w.conv2d(1, 64, 56, 56, 64, 3, 3), w.depthwise_conv2d(1, 512, 28, 28, 3, 3),
           w.gemm(128, 768, 3072)]
    slots = max(w.n_slots(s) for s in sgs)
    for lens in ([8192, 64, 4100, 1000, 68], [8191, 65, 4097, 999, 67], [8192, 64, 8193, 1000, 68]):
        seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        tiles = np.zeros((slots, int(seg[-1])), np.uint16)
        for t, sg in enumerate(sgs):
            tl, _ = w.sample_population(sg, lens[t], seed=91, stream=t)
            tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
        for flags in (0, P.REFERENCE_ROUNDING, P.FUSED_ARITHMETIC, P.REFERENCE_ROUNDING | 1, 2):
            check_prior_filter(P, sgs, seg, tiles, k, flags)
        if min(lens) >= 65:
            check_prior_filter(P, sgs, seg, tiles, 65, P.REFERENCE_ROUNDING)
    # copies of one schedule: every score equal, the k lowest indices win
    tiles[:, : lens[0]] = tiles[:, :1]
    check_prior_filter(P, sgs, seg, tiles, k, P.REFERENCE_ROUNDING)


# ---- latent schedule explorer --------------------------------------------------------------------------------------

def lse_population(sgs, lens, seed):
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = max(w.n_slots(s) for s in sgs)
    tiles = np.zeros((rows, int(seg[-1])), np.uint16)
    for t, sg in enumerate(sgs):
        tl, _ = w.sample_population(sg, lens[t], seed=seed, stream=t)
        tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
    return seg, tiles


def check_lse_against_oracle(P, sgs, seg, tiles, k, steps, seed, q16):
    """Under reference rounding every integer the loop produces equals the oracle's: the population, S_spec's
    schedules and counts; the scores bit for bit."""
    opop, oscore, ospec_t, ospec_s, ospec_n = oracle.lse(sgs, seg, tiles, k, steps, seed, q16)
    pop = dev(tiles)
    score, spec_t, spec_s, spec_n = P.lse(sgs, seg, pop, k, steps, seed, q16, flags=P.REFERENCE_ROUNDING)
    torch.cuda.synchronize()
    assert np.array_equal(spec_n.cpu().numpy(), ospec_n)
    assert np.array_equal(spec_s.cpu().numpy().view(np.uint32), ospec_s.view(np.uint32))
    assert np.array_equal(spec_t.cpu().numpy(), ospec_t)
    assert np.array_equal(score.cpu().numpy().view(np.uint32), oscore.view(np.uint32))
    gpop = pop.cpu().numpy()
    for t, sg in enumerate(sgs):
        n_slots = w.n_slots(sg)
        assert np.array_equal(gpop[:n_slots, seg[t]:seg[t + 1]], opop[:n_slots, seg[t]:seg[t + 1]])
        assert np.array_equal(gpop[n_slots:, seg[t]:seg[t + 1]], tiles[n_slots:, seg[t]:seg[t + 1]])   # rows it does not own: untouched


LSE_SGS = [w.gemm(96, 80, 72, hw=w.toy_device()), w.conv2d(1, 8, 12, 12, 16, 3, 3),
           w.gemm(64, 64, 64, dtype_bytes=2, hw=w.toy_device(), rd_levels=3, frag=(16, 16, 16)), w.batched_gemm(4, 32, 48, 40)]


@pytest.mark.parametrize("steps,q16", [(1, 0), (1, 65536), (2, 40000), (5, 52000)])
def test_lse_small_populations(P, steps, q16):
    seg, tiles = lse_population(LSE_SGS, [700, 601, 500, 444], seed=21)
    check_lse_against_oracle(P, LSE_SGS, seg, tiles, 24, steps, 77 + steps, q16)


def test_lse_large_selection_route_and_full_k(P):
    """One segment long enough for the large selection route and the per-class draft launches (aligned offsets),
    k = 4096 so that the union sorted in LDS has 8192 entries; copies are plentiful after the first mutation."""
    sgs = [w.gemm(512, 512, 512), w.depthwise_conv2d(1, 512, 28, 28, 3, 3)]
    seg, tiles = lse_population(sgs, [1 << 20, 140000], seed=22)
    check_lse_against_oracle(P, sgs, seg, tiles, 4096, 3, 5, 60000)


def test_lse_children_made_in_the_draft_kernels(P):
    """Above 2^20 candidates, with aligned offsets, the draft kernels of every step after the first make, store and
    score the children themselves (one launch per loop-nest class).  All five classes, the generic one included, a
    fragment GEMM with three reduction levels, slot counts that reach two, three and four 16-byte record pieces, and a
    last segment that ends two candidates into a thread's four (the pitch is padded to a multiple of 4)."""
    hw = w.Device(T_p=3.3e12, T_m=4.1e11, m_l0=96, m_l1=20000, pu_l1=3, n_l1=24, pu_l2=7, n_l2=5)
    d = lambda *t: tuple(t)
    bt = w.Subgraph("gemm_bt", 2, 1, (96, 80, 72), 4, 3, 4, (0, 0, 0),
                    (w.Buffer((d((0, 1)), d((2, 1)))), w.Buffer((d((1, 1)), d((2, 1))))), w.Buffer((d((0, 1)), d((1, 1)))), hw)
    sgs = [w.conv2d(1, 64, 56, 56, 64, 3, 3), w.gemm(512, 512, 512), bt, w.depthwise_conv2d(1, 512, 28, 28, 3, 3),
           w.batched_gemm(12, 128, 128, 64), w.gemm(64, 64, 64, dtype_bytes=2, hw=w.toy_device(), rd_levels=3, frag=(16, 16, 16)),
           w.gemm(128, 768, 3072)]
    lens = [200004, 150000, 180004, 150000, 170008, 100000, 150002]
    seg, tiles = lse_population(sgs, lens, seed=41)
    n = int(seg[-1])
    assert n >= 1 << 20 and n % 4 == 2 and all(int(o) % 4 == 0 for o in seg[:-1])
    k, steps, seed, q16 = 64, 3, 11, 55000
    opop, oscore, ospec_t, ospec_s, ospec_n = oracle.lse(sgs, seg, tiles, k, steps, seed, q16)
    padded = np.full((tiles.shape[0], n + 2), 7, np.uint16)
    padded[:, :n] = tiles
    pop = dev(padded)
    score, spec_t, spec_s, spec_n = P.lse(sgs, seg, pop, k, steps, seed, q16, flags=P.REFERENCE_ROUNDING)
    torch.cuda.synchronize()
    assert np.array_equal(spec_n.cpu().numpy(), ospec_n)
    assert np.array_equal(spec_s.cpu().numpy().view(np.uint32), ospec_s.view(np.uint32))
    assert np.array_equal(spec_t.cpu().numpy(), ospec_t)
    assert np.array_equal(score.cpu().numpy()[:n].view(np.uint32), oscore.view(np.uint32))
    gpop = pop.cpu().numpy()
    assert np.all(gpop[:, n:] == 7)                                                        # the padding columns: untouched
    for t, sg in enumerate(sgs):
        n_slots = w.n_slots(sg)
        assert np.array_equal(gpop[:n_slots, seg[t]:seg[t + 1]], opop[:n_slots, seg[t]:seg[t + 1]])
        assert np.array_equal(gpop[n_slots:, seg[t]:seg[t + 1]], tiles[n_slots:, seg[t]:seg[t + 1]])


def test_lse_default_arithmetic_invariants(P):
    seg, tiles = lse_population(LSE_SGS, [4000, 3000, 2000, 1000], seed=23)
    k = 64
    pop = dev(tiles)
    score, spec_t, spec_s, spec_n = P.lse(LSE_SGS, seg, pop, k, 4, 9, 50000)
    torch.cuda.synchronize()
    gpop, spec_t, spec_s, spec_n = pop.cpu().numpy(), spec_t.cpu().numpy(), spec_s.cpu().numpy(), spec_n.cpu().numpy()
    first_s, _, _ = oracle.draft_score(LSE_SGS, seg, tiles)
    for t, sg in enumerate(LSE_SGS):
        n_slots, cnt = w.n_slots(sg), int(spec_n[t])
        cols = gpop[:, seg[t]:seg[t + 1]]
        for a in range(sg.n_sp + sg.n_rd):
            lv = 4 if a < sg.n_sp else sg.rd_levels
            base = a * 4 if a < sg.n_sp else sg.n_sp * 4 + (a - sg.n_sp) * sg.rd_levels
            assert np.all(np.prod(cols[base:base + lv].astype(np.int64), axis=0) == sg.extent[a])
        block = spec_t[:n_slots, t * k:t * k + cnt]
        assert cnt >= 1 and len({tuple(c) for c in block.T}) == cnt                       # no schedule twice
        assert np.all(spec_s[t, :cnt - 1] >= spec_s[t, 1:cnt]) and np.all(np.isneginf(spec_s[t, cnt:]))
        _, o64, _ = oracle.draft_score([sg], [0, cnt], block)                             # each score belongs to its schedule
        assert np.max(np.abs(spec_s[t, :cnt] - o64) / np.abs(o64)) <= FUSED_TOL
        # exploring never loses the best schedule seen: the initial population's best is still matched or beaten
        best0 = first_s[seg[t]:seg[t + 1]].max()
        assert spec_s[t, 0] >= best0 - abs(best0) * 1e-5


# ---- the whole path ---------------------------------------------------------------------------------------------------

def run_path(P, wl, m, flags=0):
    """draft -> top-k -> (features of the drafted set, made on the host from their ids) -> verify -> top-k."""
    score = P.draft_score(wl.subgraphs, wl.seg_off, dev(wl.tiles), flags=flags)
    idx, _ = P.topk(score, wl.seg_off, wl.k_draft)
    ids = idx.cpu().numpy()
    n_stmt = np.repeat(np.array(wl.n_stmt, np.int32), wl.k_draft)
    feat = w.make_statement_features(ids.reshape(-1), n_stmt, seed=wl.seed)
    vs = P.verify_score(dev(feat), dev(n_stmt), gpu_weights(m))
    seg2 = np.arange(len(wl.subgraphs) + 1, dtype=np.int64) * wl.k_draft
    fin, _ = P.topk(vs, seg2, wl.k_final)
    torch.cuda.synchronize()
    return score.cpu().numpy(), ids, feat, n_stmt, vs.cpu().numpy(), fin.cpu().numpy(), seg2


def check_selection_within_tolerance(got, want, ref, tol):
    """Two top-k lists (candidate ids) taken on scores that differ by rounding: whatever one has and the other lacks
    must sit at the cut, i.e. within the score tolerance of the reference's k-th value."""
    for s in range(got.shape[0]):
        diff = set(got[s].tolist()) ^ set(want[s].tolist())
        cut = ref[want[s, -1]]
        for i in diff:
            assert abs(ref[i] - cut) <= 2 * tol[i], (s, i, ref[i], cut)


@pytest.mark.parametrize("mode", [4, 8, 0])
@pytest.mark.parametrize("idx,scale", [(3, 1.0), (4, 1 / 16)])
def test_whole_path(P, idx, scale, mode):
    wl = w.make_config(idx, scale=scale)
    m = w.make_mlp_weights(seed=1)
    g32, ids, feat, n_stmt, gvs, gfin, seg2 = run_path(P, wl, m, mode)
    o32, o64, _ = oracle.draft_score(wl.subgraphs, wl.seg_off, wl.tiles)
    oids, _ = oracle.topk(o32, wl.seg_off, wl.k_draft)
    if mode == P.REFERENCE_ROUNDING or (mode == 0 and wl.n < (1 << 20)):
        # draft + selection: identical to the oracle, index by index
        assert np.array_equal(ids, oids)
    else:
        # selection is exact on the library's own scores; against the oracle's scores it may differ at the cut only
        sids, _ = oracle.topk(g32, wl.seg_off, wl.k_draft)
        assert np.array_equal(ids, sids)
        check_selection_within_tolerance(ids, oids, o64, FUSED_TOL * np.abs(o64))
    # verify scores within tolerance
    ovs, _, omag = oracle.verify(feat, n_stmt, m, want_mag=True)
    tol = oracle.verify_tolerance(ovs, omag)
    assert np.all(np.abs(gvs - ovs) <= tol)
    # final selection: exact on the library's own scores ...
    sfin, _ = oracle.topk(gvs, seg2, wl.k_final)
    assert np.array_equal(gfin, sfin)
    # ... and against the oracle's scores any disagreement must sit inside the score tolerance at the cut
    ofin, _ = oracle.topk(ovs, seg2, wl.k_final)
    check_selection_within_tolerance(gfin, ofin, ovs, tol)


@pytest.mark.parametrize("idx,scale", [(3, 1.0), (4, 1 / 16)])
def test_step_replayed_from_a_captured_graph(P, idx, scale):
    """One step (PriorFilter, verify, final selection; workspaces and outputs allocated beforehand) captured into a HIP
    graph: tables travel as kernel arguments and scratch is cleared by kernels, so every replay must give the eager
    result, with eager work and synchronisations between the replays and the outputs wiped before each."""
    wl = w.make_config(idx, scale=scale)
    m = gpu_weights(w.make_mlp_weights(seed=1))
    n, n_sg = wl.n, len(wl.subgraphs)
    csg = P.to_c_subgraphs(wl.subgraphs)
    tiles = dev(wl.tiles)
    score = torch.empty(n, dtype=torch.float32, device="cuda")
    idx_d = torch.empty((n_sg, wl.k_draft), dtype=torch.int32, device="cuda")
    ws1 = torch.empty(P.workspace_bytes(P.WS_PRIOR_FILTER, n, n_sg, wl.k_draft), dtype=torch.uint8, device="cuda")
    P.prior_filter(csg, wl.seg_off, tiles, wl.k_draft, score=score, idx_out=idx_d, want_values=False, workspace=ws1)
    torch.cuda.synchronize()
    n_stmt_h = np.repeat(np.array(wl.n_stmt, np.int32), wl.k_draft)
    feat = dev(w.make_statement_features(idx_d.cpu().numpy().reshape(-1), n_stmt_h, seed=wl.seed))
    n_stmt = dev(n_stmt_h)
    n_d = n_sg * wl.k_draft
    vscore = torch.empty(n_d, dtype=torch.float32, device="cuda")
    seg2 = np.arange(n_sg + 1, dtype=np.int64) * wl.k_draft
    fin = torch.empty((n_sg, wl.k_final), dtype=torch.int32, device="cuda")
    ws2 = torch.empty(max(P.workspace_bytes(P.WS_VERIFY, n_d, 0, 0), 256), dtype=torch.uint8, device="cuda")
    ws3 = torch.empty(P.workspace_bytes(P.WS_TOPK, n_d, n_sg, wl.k_final), dtype=torch.uint8, device="cuda")

    def step():
        P.prior_filter(csg, wl.seg_off, tiles, wl.k_draft, score=score, idx_out=idx_d, want_values=False, workspace=ws1)
        P.verify_score(feat, n_stmt, m, vscore=vscore, workspace=ws2)
        P.topk(vscore, seg2, wl.k_final, idx_out=fin, want_values=False, workspace=ws3)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (score, idx_d, vscore, fin)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                      # (kernels loaded and attributes set before the capture)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (score, idx_d, vscore, fin):
            t.zero_()
        P.draft_score(csg, wl.seg_off, tiles)       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((score, idx_d, vscore, fin), want):
            assert torch.equal(got.view(torch.int32), ref.view(torch.int32)), replay


@pytest.mark.parametrize("lens,per_class", [([300000, 40000], False), ([800000, 400000], True)])
def test_timing_hook_brackets_the_largest_launch(P, lens, per_class):
    """the measurement hook: events recorded around one draft kernel launch, algorithmic bytes of that launch; results
    unchanged.  Below 2^20 candidates a call is one launch; above, one per loop-nest class."""
    import ctypes
    sgs = [w.gemm(512, 512, 512), w.conv2d(1, 64, 56, 56, 64, 3, 3)]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = max(w.n_slots(s) for s in sgs)
    tiles = P.random_init(sgs, seg, rows, 1)
    plain = P.draft_score(sgs, seg, tiles)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(), e1.record()
    torch.cuda.synchronize()
    got = ctypes.c_int64(-1)
    P.time_dominant_draft_launch(e0, e1, got)
    try:
        timed = P.draft_score(sgs, seg, tiles)
        torch.cuda.synchronize()
    finally:
        P.time_dominant_draft_launch(None, None)
    per_segment = [lens[t] * (2 * w.n_slots(sgs[t]) + 4) for t in range(2)]
    assert got.value == (per_segment[0] if per_class else sum(per_segment))   # the GEMM class holds the most candidates
    assert 0.0 < e0.elapsed_time(e1) < 50.0
    assert torch.equal(plain, timed)
    got.value = -1
    P.draft_score(sgs, seg, tiles)                                       # hook off: nothing is written
    torch.cuda.synchronize()
    assert got.value == -1


# ---- RandomInitSch (Alg. 1, Alg. 2) -----------------------------------------------------------------------------------

def _axis_slices(sg):
    out, slot = [], 0
    for a in range(sg.n_sp + sg.n_rd):
        lv = 4 if a < sg.n_sp else sg.rd_levels
        frag = 1
        if sg.frag[0]:
            frag = {sg.n_sp - 2: sg.frag[0], sg.n_sp - 1: sg.frag[1], sg.n_sp + sg.n_rd - 1: sg.frag[2]}.get(a, 1)
        out.append((slot, lv, sg.extent[a], frag))
        slot += lv
    return out


@pytest.mark.parametrize("lens", [[1000, 257, 4099], [1, 0, 70001]])
def test_random_init_matches_the_oracle(P, lens):
    """bit for bit, ragged segments (one empty), a pitch wider than the population, a spare row that must be cleared,
    columns beyond the population untouched"""
    sgs = [w.gemm(96, 80, 72, hw=w.toy_device()), w.conv2d(1, 8, 12, 12, 16, 3, 3),
           w.gemm(64, 128, 96, dtype_bytes=2, hw=w.toy_device(), rd_levels=3, frag=(16, 16, 16))]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n, rows = int(seg[-1]), max(w.n_slots(s) for s in sgs) + 1
    want = oracle.random_init(sgs, seg, rows, seed=77)
    tiles = torch.full((rows, n + 5), 0xFFFF, dtype=torch.uint16, device="cuda")
    P.random_init(sgs, seg, rows, 77, tiles=tiles)
    torch.cuda.synchronize()
    got = tiles.cpu().numpy()
    assert np.array_equal(got[:, :n], want)
    assert (got[:, n:] == 0xFFFF).all()
    # another seed gives another population; the same seed the same one
    again = P.random_init(sgs, seg, rows, 77).cpu().numpy()
    other = P.random_init(sgs, seg, rows, 78).cpu().numpy()
    assert np.array_equal(again, want) and (other != want).any()


def test_random_init_feeds_the_explorer_loop(P):
    """the generated population is a valid S_x: the loop runs on it and matches the oracle's loop on the oracle's population"""
    sgs = [w.gemm(96, 80, 72, hw=w.toy_device()), w.conv2d(1, 8, 12, 12, 16, 3, 3)]
    seg = np.array([0, 3000, 5000], np.int64)
    rows = max(w.n_slots(s) for s in sgs)
    tiles = P.random_init(sgs, seg, rows, 5)
    torch.cuda.synchronize()
    host = tiles.cpu().numpy()
    assert np.array_equal(host, oracle.random_init(sgs, seg, rows, 5))
    check_lse_against_oracle(P, sgs, seg, host, 64, 2, 9, 40000)


def test_random_init_full_size_population(P):
    """config 4's shape (16M + 4M candidates): every schedule valid; prefixes of both segments against the oracle"""
    wl = w.make_config(4)
    rows = max(w.n_slots(s) for s in wl.subgraphs)
    tiles = P.random_init(wl.subgraphs, wl.seg_off, rows, 2024)
    torch.cuda.synchronize()
    n0 = int(wl.seg_off[1])
    for t, sg in enumerate(wl.subgraphs):
        lo, hi = int(wl.seg_off[t]), int(wl.seg_off[t + 1])
        for slot, lv, extent, frag in _axis_slices(sg):
            cols = tiles[slot:slot + lv, lo:hi].to(torch.int64)
            assert bool((cols.prod(dim=0) == extent).all()) and bool((cols >= 1).all())
            assert bool((cols[lv - 1] % frag == 0).all())
        if w.n_slots(sg) < rows:
            assert bool((tiles[w.n_slots(sg):, lo:hi] == 0).all())
    m = 50000
    want = oracle.random_init(wl.subgraphs, np.array([0, n0, n0 + m], np.int64), rows, 2024)
    got = tiles.cpu().numpy()
    assert np.array_equal(got[:, :m], want[:, :m])
    assert np.array_equal(got[:, n0:n0 + m], want[:, n0:n0 + m])
    # the space is sampled, not collapsed: m uniform draws from a space of S schedules hold about S (1 - exp(-m / S))
    # distinct ones
    sg0 = wl.subgraphs[0]
    space = float(np.prod([oracle.axis_space(sg0, a) for a in range(sg0.n_sp + sg0.n_rd)]))
    distinct = len(np.unique(got[:w.n_slots(sg0), :m].T, axis=0))
    assert distinct > 0.95 * space * (1.0 - np.exp(-m / space))


def test_lse_full_size_population(P):
    """The explorer loop in the shape the benchmark times: config 4 (16M + 4M candidates, k = 4096), three steps, the
    children of steps 1 and 2 made inside the draft kernels.  What holds at any size: every schedule of the final
    population is valid; S_spec holds distinct schedules, best first, each with the oracle's C_SA of that schedule
    bit for bit; the best schedule of the initial population is matched or beaten."""
    wl = w.make_config(4)
    rows = max(w.n_slots(s) for s in wl.subgraphs)
    k = wl.k_draft
    pop = P.random_init(wl.subgraphs, wl.seg_off, rows, 99)
    first = P.draft_score(wl.subgraphs, wl.seg_off, pop, flags=P.REFERENCE_ROUNDING)
    best0 = [float(first[int(wl.seg_off[t]):int(wl.seg_off[t + 1])].max()) for t in range(len(wl.subgraphs))]
    del first
    score, spec_t, spec_s, spec_n = P.lse(wl.subgraphs, wl.seg_off, pop, k, 3, 5, 52000, flags=P.REFERENCE_ROUNDING)
    torch.cuda.synchronize()
    for t, sg in enumerate(wl.subgraphs):
        lo, hi = int(wl.seg_off[t]), int(wl.seg_off[t + 1])
        for slot, lv, extent, frag in _axis_slices(sg):
            cols = pop[slot:slot + lv, lo:hi].to(torch.int64)
            assert bool((cols.prod(dim=0) == extent).all()) and bool((cols >= 1).all())
            assert bool((cols[lv - 1] % frag == 0).all())
            del cols
        if w.n_slots(sg) < rows:
            assert bool((pop[w.n_slots(sg):, lo:hi] == 0).all())
    assert bool(torch.isfinite(score).all())
    spec_t, spec_s, spec_n = spec_t.cpu().numpy(), spec_s.cpu().numpy(), spec_n.cpu().numpy()
    for t, sg in enumerate(wl.subgraphs):
        n_slots, cnt = w.n_slots(sg), int(spec_n[t])
        block = spec_t[:n_slots, t * k:t * k + cnt]
        assert 1 <= cnt <= k and len({tuple(c) for c in block.T}) == cnt
        assert np.all(spec_s[t, :cnt - 1] >= spec_s[t, 1:cnt]) and np.all(np.isneginf(spec_s[t, cnt:]))
        o32, _, _ = oracle.draft_score([sg], [0, cnt], np.ascontiguousarray(block))
        assert np.array_equal(spec_s[t, :cnt].view(np.uint32), o32.view(np.uint32))
        assert spec_s[t, 0] >= best0[t]


# ---- the whole Pattern-aware Transformer (Sec. 4.2) ---------------------------------------------------------------------

def gpu_pacm(m):
    return {k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in m.items()}


def pacm_tolerance(want):
    """2e-2 relative, plus 5e-3 of the output range: the two sides round the same operands to bfloat16, and almost every
    candidate agrees to binary32 rounding; but when the order of a binary32 accumulation moves an entry of a pooled vector
    (magnitudes up to 64, a bfloat16 step of up to 0.5) across a rounding boundary, the head's output moves by about
    0.5 x |Wh| x |wo| x sqrt(256) ~ 1e-2 absolute, whatever its own size.  (The oracle's binary32 and binary64 results differ
    by up to 1e-2 of the range for the same reason.)"""
    return 2e-2 * np.abs(want) + 5e-3 * max(float(np.abs(want).max()), 1e-30)


def check_pacm(P, feat, n_stmt, flow, n_blk, m, label=""):
    got = P.pacm_score(dev(feat), dev(np.asarray(n_stmt, np.int32)), dev(flow), dev(np.asarray(n_blk, np.int32)), gpu_pacm(m))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    want, want64 = oracle.pacm(feat, n_stmt, flow, n_blk, m)
    assert np.isfinite(got).all(), label
    excess = np.abs(got - want) - pacm_tolerance(want)
    assert excess.max() <= 0, (label, float(excess.max()), int(excess.argmax()))
    # and the bulk agrees far more closely: the median difference is binary32 rounding
    assert np.median(np.abs(got - want)) <= 1e-5 * max(float(np.abs(want).max()), 1e-30), label
    return got, want


def test_pacm_hand_sized_dataflow_branch(P):
    """the hand-computed case of the oracle's pins, through the kernels: uniform attention, v_d = 3 sum of the embeddings"""
    bfb = w.f32_to_bf16_bits
    z = lambda *s: np.zeros(s, np.float32)
    We, Wv, Wo, Wh, wo, bh = z(64, 23), z(64, 64), z(64, 64), z(256, 320), z(256), z(256)
    We[0, 0] = We[1, 1] = 1.0
    Wv[0, 0] = Wv[1, 1] = 1.0
    Wo[0, 0] = Wo[1, 1] = 2.0
    Wh[0, 256], Wh[0, 257], bh[0], wo[0] = 1.0, -1.0, 1.0, 2.0
    m = {"W1": bfb(z(256, 164)), "b1": z(256), "W2": bfb(z(256, 256)), "b2": z(256), "We": bfb(We), "be": z(64), "Wq": bfb(z(64, 64)),
         "Wk": bfb(z(64, 64)), "Wv": bfb(Wv), "Wo": bfb(Wo), "Wh": bfb(Wh), "bh": bh, "wo": bfb(wo), "bo": -0.5}
    flow = np.zeros((2, 8, 23), np.float32)
    flow[0, 0, :2], flow[0, 1, :2], flow[0, 2, :2] = (1, 2), (3, 0), (4, 1)
    flow[1, 0, :2] = (5, 1)
    flow[1, 1, :2] = (100, -7)                                                   # beyond n_blk: ignored
    got, want = check_pacm(P, np.zeros((2, 8, 164), np.float32), [0, 0], flow, [3, 1], m)
    assert list(want) == [31.5, 25.5] and np.allclose(got, [31.5, 25.5], rtol=1e-6)


def test_pacm_random_weights_ragged_counts(P):
    m = w.make_pacm_weights(seed=1)
    rng = np.random.default_rng(8)
    for n_d in (1, 7, 8, 9, 65, 333, 2048 + 5):
        n_stmt = rng.integers(0, 9, size=n_d).astype(np.int32)
        n_blk = rng.integers(0, 9, size=n_d).astype(np.int32)
        ids = np.arange(n_d) * 31 + 5
        feat = w.make_statement_features(ids, n_stmt, pad_value=1e6)            # garbage in the rows beyond the counts
        flow = w.make_flow_features(ids, n_blk, pad_value=np.float32("nan"))
        check_pacm(P, feat, n_stmt, flow, n_blk, m, label=str(n_d))


def test_pacm_degenerate_counts(P):
    m = w.make_pacm_weights(seed=3)
    n_d = 70
    ids = np.arange(n_d)
    for n_stmt, n_blk in ((np.zeros(n_d, np.int32), np.zeros(n_d, np.int32)), (np.full(n_d, 8, np.int32), np.full(n_d, 8, np.int32)),
                          (np.zeros(n_d, np.int32), np.full(n_d, 1, np.int32)), (np.full(n_d, 1, np.int32), np.zeros(n_d, np.int32))):
        feat = w.make_statement_features(ids, n_stmt, pad_value=-3e5)
        flow = w.make_flow_features(ids, n_blk, pad_value=7e4)
        got, want = check_pacm(P, feat, n_stmt, flow, n_blk, m)
    # counts outside 0..8 are clamped
    wild_s, wild_b = np.full(n_d, 11, np.int32), np.full(n_d, -2, np.int32)
    feat = w.make_statement_features(ids, np.full(n_d, 8), pad_value=0.0)
    flow = w.make_flow_features(ids, np.zeros(n_d, np.int64))
    a = P.pacm_score(dev(feat), dev(wild_s), dev(flow), dev(wild_b), gpu_pacm(m)).cpu().numpy()
    b = P.pacm_score(dev(feat), dev(np.full(n_d, 8, np.int32)), dev(flow), dev(np.zeros(n_d, np.int32)), gpu_pacm(m)).cpu().numpy()
    assert np.array_equal(a, b)


def test_pacm_drafted_set_of_the_benchmark(P):
    """8192 candidates (config 4's drafted set), the statement counts of its two subgraphs, five to eight blocks each"""
    m = w.make_pacm_weights(seed=1)
    n_d = 8192
    ids = np.arange(n_d) * 3 + 1
    n_stmt = np.repeat(np.array([5, 4], np.int32), 4096)
    n_blk = (5 + ids % 4).astype(np.int32)
    feat = w.make_statement_features(ids, n_stmt)
    flow = w.make_flow_features(ids, n_blk)
    got = P.pacm_score(dev(feat), dev(n_stmt), dev(flow), dev(n_blk), gpu_pacm(m)).cpu().numpy()
    pick = np.unique(np.concatenate([np.arange(0, 64), np.arange(n_d - 64, n_d), np.random.default_rng(2).integers(0, n_d, 400)]))
    want, _ = oracle.pacm(feat[pick], n_stmt[pick], flow[pick], n_blk[pick], m)
    assert np.all(np.abs(got[pick] - want) <= pacm_tolerance(want))
    assert np.median(np.abs(got[pick] - want)) <= 1e-5 * np.abs(want).max()


# ---- momentum online adaptation (Sec. 4.3) -----------------------------------------------------------------------------

@pytest.mark.parametrize("n,offset", [(107777, 0), (4099, 1), (3, 0), (256 * 164 + 256 + 256 * 256 + 256 + 256, 0)])
def test_moa_update_matches_the_oracle(P, n, offset):
    """bit for bit in binary32 and in the bfloat16 copy; aligned (four-wide with a tail) and unaligned calls; values with
    subnormals and exact ties of the bfloat16 rounding"""
    rng = np.random.default_rng(n)
    s = rng.uniform(-0.1, 0.1, n).astype(np.float32)
    t = (s + rng.normal(0, 1e-3, n)).astype(np.float32)
    s[:3] = [1.00390625, 3.0e-39, -1.01171875][:min(3, n)]
    t[:3] = s[:3]
    for m in (0.99, 1.0, 0.0, 0.5):
        want, want_bf, f64 = oracle.moa_update(s, t, m)
        buf_s = torch.zeros(n + offset, dtype=torch.float32, device="cuda")
        buf_t = torch.zeros(n + offset, dtype=torch.float32, device="cuda")
        buf_b = torch.full((n + offset,), 0xFFFF, dtype=torch.uint16, device="cuda")
        gs, gt, gb = buf_s[offset:], buf_t[offset:], buf_b[offset:]
        gs.copy_(torch.from_numpy(s)), gt.copy_(torch.from_numpy(t))
        P.moa_update(gs, gt, m, bf16=gb)
        torch.cuda.synchronize()
        assert np.array_equal(gs.cpu().numpy().view(np.uint32), want.view(np.uint32)), m
        assert np.array_equal(gb.cpu().numpy(), want_bf), m
        assert np.abs(gs.cpu().numpy() - f64).max() <= 2 * np.spacing(np.float32(1.02))
        if offset:
            assert int(buf_b[0]) == 0xFFFF and float(buf_s[0]) == 0.0        # nothing before the first element is touched
        # without the bfloat16 copy
        gs.copy_(torch.from_numpy(s))
        P.moa_update(gs, gt, m)
        torch.cuda.synchronize()
        assert np.array_equal(gs.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_moa_update_feeds_the_verify_stage(P):
    """the bfloat16 copy of an adapted W1 is what pruner_verify_score then computes with"""
    m = w.make_mlp_weights(seed=1)
    rng = np.random.default_rng(4)
    master = {k: w.bf16_bits_to_f32(m[k]).astype(np.float32) for k in ("W1", "W2", "w3")}
    target = {k: (v + rng.normal(0, 2e-3, v.shape)).astype(np.float32) for k, v in master.items()}
    new = dict(m)
    gm = {k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in m.items()}
    for k in master:
        _, bits, _ = oracle.moa_update(master[k], target[k], 0.99)
        new[k] = bits.reshape(m[k].shape)
        gs, gt = dev(master[k].ravel()), dev(target[k].ravel())
        gb = torch.empty(gs.numel(), dtype=torch.uint16, device="cuda")
        P.moa_update(gs, gt, 0.99, bf16=gb)
        gm[k] = gb.reshape(m[k].shape)
    n_d = 300
    n_stmt = (3 + np.arange(n_d) % 6).astype(np.int32)
    feat = w.make_statement_features(np.arange(n_d), n_stmt, seed=3)
    got = P.verify_score(dev(feat), dev(n_stmt), gm)
    torch.cuda.synchronize()
    want, _, mag = oracle.verify(feat, n_stmt, new, want_mag=True)
    assert np.all(np.abs(got.cpu().numpy() - want) <= oracle.verify_tolerance(want, mag))
    for k in master:
        assert np.array_equal(gm[k].cpu().numpy(), new[k])


def test_prior_filter_long_and_short_segments_together(P):
    """the selection's large route with segments from 64 to 1.3 M candidates in one call (k equal to the shortest), and
    the draft kernel's per-class launches with a class that appears twice"""
    sgs = [w.gemm(512, 512, 512), w.conv2d(1, 64, 56, 56, 64, 3, 3), w.gemm(128, 768, 3072), w.depthwise_conv2d(1, 512, 28, 28, 3, 3),
           w.batched_gemm(12, 128, 128, 64)]
    lens = [1300000, 300, 70000, 900000, 64]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = max(w.n_slots(s) for s in sgs)
    host = P.random_init(sgs, seg, rows, 21).cpu().numpy()
    check_prior_filter(P, sgs, seg, host, 64, P.REFERENCE_ROUNDING)
    check_prior_filter(P, sgs, seg, host, 64, 0)


def test_maximum_number_of_subgraphs(P):
    """PRUNER_MAX_SUBGRAPHS segments (tables far larger than one upload launch carries; segments of 17 to 56 candidates,
    some shorter than a vector): RandomInitSch, PriorFilter and two steps of the explorer loop against the oracle."""
    n_sg = 4096
    shapes = w.bert_base_subgraphs(6)
    sgs = [shapes[t % 6] for t in range(n_sg)]
    lens = [17 + (t * 7) % 40 for t in range(n_sg)]
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = max(w.n_slots(s) for s in sgs)
    tiles = P.random_init(sgs, seg, rows, 12)
    torch.cuda.synchronize()
    host = tiles.cpu().numpy()
    assert np.array_equal(host, oracle.random_init(sgs, seg, rows, 12))
    check_prior_filter(P, sgs, seg, host, 16, P.REFERENCE_ROUNDING)
    check_prior_filter(P, sgs, seg, host, 16, 0)
    check_lse_against_oracle(P, sgs, seg, host, 16, 2, 3, 40000)


def test_full_size_stress_population_in_the_benchmark_configuration(P):
    """Config 4 at full size (16M + 4M candidates), launched as bench.py launches it (pruner_prior_filter): every
    draft score and the draft selection against the oracle; then the same under reference rounding, bit for bit."""
    wl = w.make_config(4)
    o32, o64, _ = oracle.draft_score(wl.subgraphs, wl.seg_off, wl.tiles)
    tiles = dev(wl.tiles)
    score, idx, val = P.prior_filter(wl.subgraphs, wl.seg_off, tiles, wl.k_draft)
    torch.cuda.synchronize()
    g32 = score.cpu().numpy()
    assert (np.abs(g32 - o64) / np.abs(o64)).max() <= FUSED_TOL
    si, sv = oracle.topk(g32, wl.seg_off, wl.k_draft)
    assert np.array_equal(idx.cpu().numpy(), si) and np.array_equal(val.cpu().numpy(), sv)
    oi, ov = oracle.topk(o32, wl.seg_off, wl.k_draft)
    check_selection_within_tolerance(idx.cpu().numpy(), oi, o64, FUSED_TOL * np.abs(o64))
    # on this population the fused form's selection IS the oracle's, row by row (a measured fact of these seeded
    # inputs, asserted so that a change shows; what holds for any input is the check above)
    assert np.array_equal(idx.cpu().numpy(), oi)

    score, idx, val = P.prior_filter(wl.subgraphs, wl.seg_off, tiles, wl.k_draft, flags=P.REFERENCE_ROUNDING)
    torch.cuda.synchronize()
    g32 = score.cpu().numpy()
    assert np.array_equal(g32.view(np.uint32), o32.view(np.uint32))
    assert (np.abs(g32 - o64) / np.abs(o64)).max() <= 1e-5
    assert np.array_equal(idx.cpu().numpy(), oi) and np.array_equal(val.cpu().numpy(), ov)

    # the two separate calls give the same rows
    s2 = P.draft_score(wl.subgraphs, wl.seg_off, tiles, flags=P.REFERENCE_ROUNDING)
    i2, v2 = P.topk(s2, wl.seg_off, wl.k_draft)
    torch.cuda.synchronize()
    assert np.array_equal(i2.cpu().numpy(), oi) and np.array_equal(v2.cpu().numpy(), ov)


# sizes of the symmetric difference between the fused form's draft selection and the oracle's, per configuration (all
# subgraphs together), as measured on these seeded populations; config 4 at full size is in the test above
FUSED_SELECTION_DIFFERENCE = {0: 0, 1: 0, 2: 10, 3: 10}


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_draft_selection_against_the_oracle_on_every_configuration(P, idx):
    """Draft top-k of the configurations at full size against the oracle's selection on its own binary32 scores.
    Without a switch (these populations run as one launch, i.e. with reference rounding) and under
    PRUNER_REFERENCE_ROUNDING: the same lists, row by row.  Under PRUNER_FUSED_ARITHMETIC: the size of the symmetric
    difference is recorded above and asserted, and every candidate in it lies within the score tolerance of the cut."""
    wl = w.make_config(idx)
    o32, o64, _ = oracle.draft_score(wl.subgraphs, wl.seg_off, wl.tiles)
    oi, ov = oracle.topk(o32, wl.seg_off, wl.k_draft)
    tiles = dev(wl.tiles)
    for flags in (0, P.REFERENCE_ROUNDING):
        _, gi, gv = P.prior_filter(wl.subgraphs, wl.seg_off, tiles, wl.k_draft, flags=flags)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(gv.cpu().numpy().view(np.uint32), ov.view(np.uint32))
    _, gi, _ = P.prior_filter(wl.subgraphs, wl.seg_off, tiles, wl.k_draft, flags=P.FUSED_ARITHMETIC)
    gi = gi.cpu().numpy()
    diff = sum(len(set(a.tolist()) ^ set(b.tolist())) for a, b in zip(gi, oi))
    print(f"config {idx}: fused-arithmetic selection differs from the oracle's in {diff} of {oi.size} candidates")
    assert diff == FUSED_SELECTION_DIFFERENCE[idx]
    check_selection_within_tolerance(gi, oi, o64, FUSED_TOL * np.abs(o64))


# ---- one whole round of Alg. 1: S_spec from the explorer, S_draft = S_spec U RandomInitSch, verify, S_measured ---------

def _draft_set(spec_tiles, spec_count, random_tiles, sgs, k, p0):
    """S_draft of Alg. 1 as a set per subgraph: S_spec's schedules followed by those of the p0 random schedules that are not
    among them already (nor twice among themselves).  Host-side bookkeeping on either side's arrays; returns the list of
    per-subgraph schedule lists (tuples of the subgraph's own slots)."""
    out = []
    for t, sg in enumerate(sgs):
        n_slots = w.n_slots(sg)
        members = [tuple(c) for c in spec_tiles[:n_slots, t * k:t * k + int(spec_count[t])].T.tolist()]
        seen = set(members)
        for c in random_tiles[:n_slots, t * p0:(t + 1) * p0].T.tolist():
            if tuple(c) not in seen:
                seen.add(tuple(c))
                members.append(tuple(c))
        out.append(members)
    return out


def test_one_round_with_the_union_of_explored_and_random_schedules(P):
    """Alg. 1 on a scaled BERT-shaped workload: the explorer's S_spec (two steps, reference rounding: equal to the oracle's
    bit for bit), RandomInitSch for p0 more schedules per subgraph, the set union of the two, the verify model on the
    union (features keyed by the schedule, so that a schedule has one feature row set whichever part it came from), and
    the final selection: against the oracle at every stage."""
    import zlib
    wl = w.make_config(3, scale=0.04)                      # 20 subgraphs x 2,000 candidates
    sgs, seg, k, p0, k_final = wl.subgraphs, wl.seg_off, 48, 16, 8
    rows = wl.tiles.shape[0]
    n_sg = len(sgs)
    seg_r = np.arange(n_sg + 1, dtype=np.int64) * p0
    # device side
    pop = dev(wl.tiles)
    _, g_spec_t, _, g_spec_n = P.lse(sgs, seg, pop, k, 2, 17, 40000, flags=P.REFERENCE_ROUNDING)
    g_rand = P.random_init(sgs, seg_r, rows, 23)
    torch.cuda.synchronize()
    g_draft = _draft_set(g_spec_t.cpu().numpy(), g_spec_n.cpu().numpy(), g_rand.cpu().numpy(), sgs, k, p0)
    # oracle side
    _, _, o_spec_t, _, o_spec_n = oracle.lse(sgs, seg, wl.tiles, k, 2, seed=17, mutate_q16=40000)
    o_rand = oracle.random_init(sgs, seg_r, rows, 23)
    o_draft = _draft_set(o_spec_t, o_spec_n, o_rand, sgs, k, p0)
    assert g_draft == o_draft                               # the drafted sets are the same sets in the same order
    sizes = [len(d) for d in g_draft]
    assert all(s >= k_final for s in sizes) and any(s > int(c) for s, c in zip(sizes, g_spec_n.cpu().numpy()))   # the random part adds members
    # verify stage on the union: one feature row set per schedule
    ids = np.array([zlib.crc32(np.array((t,) + sched, np.uint32).tobytes()) & 0x7FFFFFFF for t, d in enumerate(g_draft) for sched in d], np.int64)
    n_stmt = np.concatenate([np.full(len(d), wl.n_stmt[t], np.int32) for t, d in enumerate(g_draft)])
    feat = w.make_statement_features(ids, n_stmt, seed=wl.seed)
    m = w.make_mlp_weights(seed=1)
    seg2 = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    gvs = P.verify_score(dev(feat), dev(n_stmt), gpu_weights(m))
    gfin, _ = P.topk(gvs, seg2, k_final)
    torch.cuda.synchronize()
    gvs, gfin = gvs.cpu().numpy(), gfin.cpu().numpy()
    ovs, _, omag = oracle.verify(feat, n_stmt, m, want_mag=True)
    tol = oracle.verify_tolerance(ovs, omag)
    assert np.all(np.abs(gvs - ovs) <= tol)
    sfin, _ = oracle.topk(gvs, seg2, k_final)
    assert np.array_equal(gfin, sfin)                       # S_measured: exact on the library's own scores ...
    ofin, _ = oracle.topk(ovs, seg2, k_final)
    check_selection_within_tolerance(gfin, ofin, ovs, tol)  # ... and within the score tolerance of the oracle's at the cut
