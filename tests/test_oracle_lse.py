"""Pins of the oracle's latent schedule explorer (Alg. 2: C_SA, PriorFilter, SchMutation over nSteps).

The mutation operator itself is a reading (the paper names a genetic algorithm over tiling factors and gives no
operator: "parity unpinned" by the paper); what the paper and the mathematics do fix is pinned here: the random
generator against its published outputs, PriorFilter against a plain sort, and the invariants of the loop.
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
