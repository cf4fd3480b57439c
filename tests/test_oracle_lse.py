"""Pins of the oracle's latent schedule explorer (Alg. 2: C_SA, PriorFilter, SchMutation over nSteps).

The mutation operator itself is a reading (the paper names a genetic algorithm over tiling factors and gives no
operator, so no value the paper prints can pin it).  Pinned here: the random generator against its published outputs;
PriorFilter against a plain sort; the invariants of the loop; and, from outside the oracle, children, parents, hashes and
the (score, hash) order of S_spec traced step by step in plain integers from the published generator
(tests/golden/lse_trace.json), plus the distributions of the parent pick and of the moves.
"""
import numpy as np
import pytest

import oracle
import workloads as w


def test_splitmix64_published_outputs():
    # first outputs of the public-domain splitmix64.c for seed 0 and for seed 1234567
    assert [oracle.splitmix64_draw(0, c) for c in (1, 2, 3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [oracle.splitmix64_draw(1234567, c) for c in (1, 2, 3)] == [6457827717110365317, 3203168211198807973, 9817491932198370423]


def _population(sgs, lens, seed):
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = max(w.n_slots(s) for s in sgs)
    tiles = np.zeros((rows, int(seg[-1])), np.uint16)
    for t, sg in enumerate(sgs):
        tl, _ = w.sample_population(sg, lens[t], seed=seed, stream=t)
        tiles[: tl.shape[0], seg[t]:seg[t + 1]] = tl
    return seg, tiles


def _axis_products(sg, cols):
    out = []
    for a in range(sg.n_sp + sg.n_rd):
        lv = 4 if a < sg.n_sp else sg.rd_levels
        base = a * 4 if a < sg.n_sp else sg.n_sp * 4 + (a - sg.n_sp) * sg.rd_levels
        out.append(np.prod(cols[base:base + lv].astype(np.int64), axis=0))
    return out


SGS = [w.gemm(96, 80, 72, hw=w.toy_device()), w.conv2d(1, 8, 12, 12, 16, 3, 3),
       w.gemm(64, 64, 64, dtype_bytes=2, hw=w.toy_device(), rd_levels=3, frag=(16, 16, 16))]
LENS = [700, 600, 500]


def _distinct_best(score, tiles, k):
    """The k best distinct columns: order by (score desc, position asc), a column counts once."""
    order = np.lexsort((np.arange(len(score)), -score.astype(np.float64)))
    seen, keep = set(), []
    for i in order:
        key = (float(score[i]), tuple(tiles[:, i]))
        if key not in seen:
            seen.add(key)
            keep.append(i)
            if len(keep) == k:
                break
    return keep


def _as_set(score_row, tiles_block, count):
    return {(float(score_row[r]), tuple(tiles_block[:, r])) for r in range(count)}


def test_one_step_is_prior_filter_of_the_initial_population():
    seg, tiles = _population(SGS, LENS, seed=5)
    k = 32
    pop, score, spec_tiles, spec_score, spec_count = oracle.lse(SGS, seg, tiles, k, 1, seed=7, mutate_q16=0)
    s32, _, _ = oracle.draft_score(SGS, seg, tiles)
    idx, val = oracle.topk(s32, seg, k)
    assert np.array_equal(score, s32)
    for t, sg in enumerate(SGS):
        n_slots = w.n_slots(sg)
        block = spec_tiles[:, t * k:(t + 1) * k]
        cnt = int(spec_count[t])
        # the k best of the population with copies counted once (plain definition), as a set ...
        want = {(float(val[t, r]), tuple(tiles[:n_slots, idx[t, r]])) for r in range(k)}
        assert _as_set(spec_score[t], block[:n_slots], cnt) == want and cnt == len(want)
        # ... stored best first, unused entries and rows cleared
        assert np.all(spec_score[t, :cnt - 1] >= spec_score[t, 1:cnt]) and np.all(np.isneginf(spec_score[t, cnt:]))
        assert not block[n_slots:].any() and not block[:, cnt:].any()
        # without mutation every child is a copy of a member of S_spec
        assert {tuple(c) for c in pop[:n_slots, seg[t]:seg[t + 1]].T} <= {tuple(c) for c in block[:n_slots, :cnt].T}


def test_more_steps_without_mutation_change_nothing():
    seg, tiles = _population(SGS, LENS, seed=6)
    a = oracle.lse(SGS, seg, tiles, 16, 1, seed=1, mutate_q16=0)
    b = oracle.lse(SGS, seg, tiles, 16, 4, seed=1, mutate_q16=0)
    # the later populations are copies of S_spec's members, and a schedule counts once
    for x, y in zip(a[2:], b[2:]):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("mutate_q16", [65536, 30000])
def test_loop_invariants(mutate_q16):
    seg, tiles = _population(SGS, LENS, seed=8)
    k = 24
    prev_cut = None
    for steps in (1, 2, 5):
        pop, score, spec_tiles, spec_score, spec_count = oracle.lse(SGS, seg, tiles, k, steps, seed=3, mutate_q16=mutate_q16)
        for t, sg in enumerate(SGS):
            n_slots = w.n_slots(sg)
            cols = pop[:, seg[t]:seg[t + 1]]
            # every mutation keeps the product of an axis's factors, and whole fragments stay whole
            for a, prod in enumerate(_axis_products(sg, cols)):
                assert np.all(prod == sg.extent[a])
            if sg.frag[0]:
                assert np.all(cols[(sg.n_sp - 2) * 4 + 3] % 16 == 0) and np.all(cols[(sg.n_sp - 1) * 4 + 3] % 16 == 0)
                assert np.all(cols[n_slots - 1] % 16 == 0)
            # S_spec: best first, no schedule twice, and each score is C_SA of the schedule stored with it
            cnt = int(spec_count[t])
            ss = spec_score[t, :cnt]
            block = spec_tiles[:n_slots, t * k:t * k + cnt]
            assert np.all(ss[:-1] >= ss[1:])
            assert len({tuple(c) for c in block.T}) == cnt
            again, _, _ = oracle.draft_score([sg], [0, cnt], block)
            assert np.array_equal(again, ss)
        # the k-th best fitness never gets worse with more steps (same seed: the runs share their first steps)
        cut = spec_score[:, -1].copy()
        if prev_cut is not None:
            assert np.all(cut >= prev_cut)
        prev_cut = cut
    # with mutation on, the population does move
    assert not np.array_equal(pop, tiles)


def test_second_step_is_the_set_union_with_the_k_best_of_the_mutated_population():
    """Two steps, recomputed from the one-step result with plain Python sets: S_spec after step 2 holds the k best
    distinct schedules of S_spec(step 1) U (the k best of the population after the first mutation)."""
    seg, tiles = _population(SGS[:1], LENS[:1], seed=9)
    k, sg = 20, SGS[0]
    n_slots = w.n_slots(sg)
    pop1, s1, spec1_t, spec1_s, spec1_n = oracle.lse(SGS[:1], seg, tiles, k, 1, seed=11, mutate_q16=50000)
    _, s2, spec2_t, spec2_s, spec2_n = oracle.lse(SGS[:1], seg, tiles, k, 2, seed=11, mutate_q16=50000)
    second, _, _ = oracle.draft_score(SGS[:1], seg, pop1)
    assert np.array_equal(second, s2)                                     # the second step scored the mutated population
    idx, val = oracle.topk(second, seg, k)
    union_score = np.concatenate([spec1_s[0, :spec1_n[0]], val[0]])
    union_tiles = np.concatenate([spec1_t[:n_slots, :spec1_n[0]], pop1[:n_slots, idx[0]]], axis=1)
    keep = _distinct_best(union_score, union_tiles, k)
    assert spec2_n[0] == len(keep)
    assert _as_set(spec2_s[0], spec2_t[:n_slots], spec2_n[0]) == {(float(union_score[i]), tuple(union_tiles[:, i])) for i in keep}
    assert np.array_equal(spec2_s[0, :len(keep)], union_score[keep])      # same scores in the same order


def test_bad_arguments():
    seg, tiles = _population(SGS[:1], [100], seed=1)
    with pytest.raises(oracle.OracleError):
        oracle.lse(SGS[:1], seg, tiles, 101, 1, seed=0, mutate_q16=0)     # k above the population
    with pytest.raises(oracle.OracleError):
        oracle.lse(SGS[:1], seg, tiles, 10, 0, seed=0, mutate_q16=0)
    with pytest.raises(oracle.OracleError):
        oracle.lse(SGS[:1], seg, tiles, 10, 1, seed=0, mutate_q16=65537)


# ---- cases traced outside the oracle (tests/golden/lse_trace.json, written by tests/golden/make_lse_trace.py in plain
# ---- Python integers from the published SplitMix64 definition; the script imports nothing of this repository)

def _trace():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "lse_trace.json")) as f:
        return json.load(f)["scenarios"]


def _scenario_inputs(sc):
    d = sc["subgraph"]
    sg = w.gemm(d["M"], d["N"], d["K"], dtype_bytes=d.get("dtype_bytes", 4), hw=w.toy_device(), rd_levels=d["rd_levels"],
                frag=tuple(d["frag"]))
    variants = np.array(sc["variants"], np.uint16)
    tiles = np.ascontiguousarray(variants[np.arange(sc["n"]) % len(variants)].T)
    return sg, np.array([0, sc["n"]], np.int64), tiles


@pytest.mark.parametrize("name", ["tie_gemm", "fragment_gemm"])
def test_traced_children_parents_and_hash_order(name):
    """Every stored child was derived by hand-checkable integer steps: draws -> bit fields -> parent, gate, axis, source and
    destination level, prime -> child.  A wrong bit field, a biased destination, the wrong prime, an off-by-one at the
    mutation threshold, a different counter layout or a different hash all change at least one stored child."""
    sc = _trace()[name]
    sg, seg, tiles = _scenario_inputs(sc)
    k, n_slots = sc["k"], w.n_slots(sg)
    # the scenario's schedules tie in fitness (only V * I enters the symbols), so the hash alone orders S_spec
    s32, _, _ = oracle.draft_score([sg], seg, tiles)
    assert len(set(s32.view(np.uint32).tolist())) == 1
    for run in sc["runs"]:
        pop, _, spec_tiles, spec_score, spec_count = oracle.lse([sg], seg, tiles, k, run["n_steps"], seed=sc["seed"],
                                                                mutate_q16=run["mutate_q16"])
        if run["n_steps"] == 1 or run["mutate_q16"] == 0:
            assert int(spec_count[0]) == len(sc["spec"])
            assert spec_tiles[:n_slots, :len(sc["spec"])].T.tolist() == sc["spec"], "S_spec is not in (score, hash) order"
        for kid in run["children"]:
            assert pop[:n_slots, kid["j"]].tolist() == kid["child"], (name, run["mutate_q16"], kid)


def test_traced_first_child_uses_the_published_outputs():
    """Child 0 of step 0 under seed 0 draws the first two published outputs of splitmix64.c; the fixture's decomposition of
    them is checked here digit by digit, so the fixture itself is pinned to the publication."""
    kid = _trace()["tie_gemm"]["runs"][0]["children"][0]
    assert kid["u1"] == "0xE220A8397B1DCDAF" and kid["u2"] == "0x6E789E6AA1B965F4"
    assert kid["low32_u1"] == 0x7B1DCDAF and kid["gate"] == 0xA839 and kid["fields"] == [0xF4, 0x65, 0xB9, 0xA1]
    # 0x7B1DCDAF / 2^32 = 0.4809...: member 7 of 16; 0xF4 = 244 of 256 -> the last of 3 axes; 101 of 256 -> level 0 of 2;
    # the only other level is 1; 161 of 256 -> the second of the two primes of 6
    assert (kid["parent"], kid["axis"], kid["src"], kid["dst"], kid["v"], kid["p"]) == (7, 2, 0, 1, 6, 3)
    assert [oracle.splitmix64_draw(0, c) for c in (1, 2)] == [int(kid["u1"], 16), int(kid["u2"], 16)]


def test_schedule_hash_orders_equal_scores():
    """Two distinct schedules with the same fitness: the smaller hash comes first whatever their order in the population."""
    sc = _trace()["tie_gemm"]
    sg, _, _ = _scenario_inputs(sc)
    a, b = sc["spec"][3], sc["spec"][11]                   # hash(a) < hash(b) by the fixture
    assert int(sc["spec_hash"][3], 16) < int(sc["spec_hash"][11], 16)
    for first, second in ((a, b), (b, a)):
        tiles = np.array([first, second, first, second], np.uint16).T.copy()
        _, _, spec_tiles, spec_score, spec_count = oracle.lse([sg], [0, 4], tiles, 2, 1, seed=0, mutate_q16=0)
        assert int(spec_count[0]) == 2 and spec_score[0, 0] == spec_score[0, 1]
        assert spec_tiles[:10, 0].tolist() == a and spec_tiles[:10, 1].tolist() == b


def _chi2(obs, exp):
    obs, exp = np.asarray(obs, float), np.asarray(exp, float)
    return float(((obs - exp) ** 2 / exp).sum())


def test_parent_pick_is_uniform_over_spec():
    sc = _trace()["tie_gemm"]
    sg, _, _ = _scenario_inputs(sc)
    n = 32768
    variants = np.array(sc["variants"], np.uint16)
    tiles = np.ascontiguousarray(variants[np.arange(n) % 16].T)
    pop, _, spec_tiles, _, cnt = oracle.lse([sg], [0, n], tiles, 16, 1, seed=99, mutate_q16=0)
    spec = [tuple(c) for c in spec_tiles[:10, :16].T]
    counts = np.zeros(16)
    for col in pop[:10].T:
        counts[spec.index(tuple(col))] += 1
    # 15 degrees of freedom: 99.9th percentile 37.7
    assert _chi2(counts, np.full(16, n / 16)) < 37.7


def test_moves_are_uniform_over_axis_source_destination_and_prime():
    """One parent whose ten factors are all 6 (two primes each) on a plain GEMM: every child mutates, every move is legal,
    and a move is identified by comparing child and parent.  Its distribution must be the product of uniform picks
    (up to the 1/256 granularity of an 8-bit field): axis 1/3; (source, destination) uniform over the ordered pairs of
    distinct levels; prime 1/2."""
    sg = w.gemm(6 ** 4, 6 ** 4, 36, hw=w.toy_device())
    parent = np.full(10, 6, np.uint16)
    n = 60000
    tiles = np.ascontiguousarray(np.tile(parent[:, None], (1, n)))
    pop, _, _, _, cnt = oracle.lse([sg], [0, n], tiles, 1, 1, seed=2024, mutate_q16=65536)
    assert int(cnt[0]) == 1
    seen = {}
    for col in pop[:10].T.astype(np.int64):
        lo = np.flatnonzero(col < 6)
        hi = np.flatnonzero(col > 6)
        assert len(lo) == 1 and len(hi) == 1                       # exactly one prime moved between two slots
        p = 6 // col[lo[0]]
        assert p in (2, 3) and col[hi[0]] == 6 * p
        axis_lo = lo[0] // 4 if lo[0] < 8 else 2
        axis_hi = hi[0] // 4 if hi[0] < 8 else 2
        assert axis_lo == axis_hi                                  # within one axis
        seen[(int(lo[0]), int(hi[0]), int(p))] = seen.get((int(lo[0]), int(hi[0]), int(p)), 0) + 1
    cells, exp = [], []
    for axis, (base, lv) in enumerate(((0, 4), (4, 4), (8, 2))):
        for s in range(lv):
            for d in range(lv):
                if s != d:
                    for p in (2, 3):
                        cells.append(seen.get((base + s, base + d, p), 0))
                        exp.append(n / 3 / (lv * (lv - 1)) / 2)
    assert sum(cells) == n and min(cells) > 0
    # 51 degrees of freedom (52 cells): 99.9th percentile 87.97; the 8-bit granularity shifts a cell's probability by at most
    # 1/256 of itself per field, which adds about n * 3 * (1/256)^2 = 3 to the statistic
    assert _chi2(cells, exp) < 95.0


def test_mutation_rate_follows_mutate_q16():
    sg = w.gemm(6 ** 4, 6 ** 4, 36, hw=w.toy_device())
    n = 40000
    tiles = np.full((10, n), 6, np.uint16)
    for q16 in (0, 16384, 49152, 65536):
        pop, _, _, _, _ = oracle.lse([sg], [0, n], tiles, 1, 1, seed=5, mutate_q16=q16)
        moved = int((pop != 6).any(axis=0).sum())
        p = q16 / 65536
        assert abs(moved - n * p) <= 4.5 * np.sqrt(n * p * (1 - p)) + 1e-9
