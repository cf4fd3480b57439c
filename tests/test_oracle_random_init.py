"""Pins of the oracle's RandomInitSch (Alg. 1: S_draft = S_spec U RandomInitSch(p0); Alg. 2: the initial S_x).

The paper fixes only that schedules are sampled at random from the schedule space; the numbering of the space is a
reading ("parity unpinned" by the paper).  What the mathematics fixes is pinned here: the size of the space against
the closed form and brute force, validity of every schedule, the stated numbering against brute-force enumeration,
coverage and uniformity, and independence from how the population is laid out.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
import workloads as w

MASK = (1 << 64) - 1


def _factorisations(n, levels):
    """all ordered factorisations of n into `levels` factors, by brute force"""
    if levels == 1:
        return [(n,)]
    return [(d,) + rest for d in range(1, n + 1) if n % d == 0 for rest in _factorisations(n // d, levels - 1)]


def _primes(n):
    out, p = [], 2
    while n > 1:
        e = 0
        while n % p == 0:
            n //= p
            e += 1
        if e:
            out.append((p, e))
        p += 1
    return out


def _levels(sg, a):
    return 4 if a < sg.n_sp else sg.rd_levels


def _slot0(sg, a):
    return a * 4 if a < sg.n_sp else sg.n_sp * 4 + (a - sg.n_sp) * sg.rd_levels


def _fragment(sg, a):
    if not sg.frag[0]:
        return 1
    return {sg.n_sp - 2: sg.frag[0], sg.n_sp - 1: sg.frag[1], sg.n_sp + sg.n_rd - 1: sg.frag[2]}.get(a, 1)


@pytest.mark.parametrize("n,levels,count", [(512, 4, 220), (512, 2, 10), (768, 4, 660), (3072, 4, 1144), (56, 4, 80), (64, 4, 84),
                                            (4096, 4, 455), (256, 4, 165), (28, 4, 40)])
def test_space_size_closed_form(n, levels, count):
    # ordered L-factorisations of prod p^e number prod binom(e + L - 1, L - 1)
    assert math.prod(math.comb(e + levels - 1, levels - 1) for _, e in _primes(n)) == count
    sg = w.gemm(n, 8, n, rd_levels=2) if levels == 4 else w.gemm(8, 8, n, rd_levels=2)
    assert oracle.axis_space(sg, 0 if levels == 4 else 2) == count


@pytest.mark.parametrize("n", [1, 2, 12, 36, 60, 97])
def test_space_size_brute_force(n):
    sg = w.gemm(n, 8, n, rd_levels=3)
    assert oracle.axis_space(sg, 0) == len(_factorisations(n, 4))
    assert oracle.axis_space(sg, 2) == len(_factorisations(n, 3))


SGS = [w.gemm(96, 80, 72, hw=w.toy_device()), w.conv2d(1, 8, 12, 12, 16, 3, 3),
       w.gemm(64, 128, 96, dtype_bytes=2, hw=w.toy_device(), rd_levels=3, frag=(16, 16, 16))]


def _generate(sgs, lens, seed):
    seg = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = max(w.n_slots(s) for s in sgs)
    return seg, oracle.random_init(sgs, seg, rows, seed)


def test_every_schedule_is_valid():
    seg, tiles = _generate(SGS, [500, 300, 400], seed=3)
    for t, sg in enumerate(SGS):
        cols = tiles[:, seg[t]:seg[t + 1]].astype(np.int64)
        for a in range(sg.n_sp + sg.n_rd):
            lv, b = _levels(sg, a), _slot0(sg, a)
            assert (cols[b:b + lv] >= 1).all()
            assert (np.prod(cols[b:b + lv], axis=0) == sg.extent[a]).all()
            assert (cols[b + lv - 1] % _fragment(sg, a) == 0).all()          # whole fragments innermost
        assert (cols[w.n_slots(sg):] == 0).all()                            # rows the subgraph does not own


def test_numbering_against_brute_force_enumeration():
    """candidate c, axis a: R = floor(u * count / 2^64), u = draw 8c + a + 1; R's mixed-radix digits (smallest prime
    least significant) are lexicographic ranks of the primes' compositions: rebuilt here from sorted lists."""
    seed = 11
    seg, tiles = _generate(SGS, [40, 40, 40], seed)
    for t, sg in enumerate(SGS):
        for c in range(int(seg[t]), int(seg[t + 1])):
            for a in range(sg.n_sp + sg.n_rd):
                lv, g = _levels(sg, a), _fragment(sg, a)
                pe = _primes(sg.extent[a] // g)
                comps = [sorted(x for x in itertools.product(range(e + 1), repeat=lv) if sum(x) == e) for _, e in pe]
                count = math.prod(len(cs) for cs in comps)
                u = oracle.splitmix64_draw(seed, (8 * c + a + 1) & MASK)
                R = (u * count) >> 64
                f = [1] * lv
                for (p, _), cs in zip(pe, comps):
                    x = cs[R % len(cs)]
                    R //= len(cs)
                    for l in range(lv):
                        f[l] *= p ** x[l]
                f[-1] *= g
                b = _slot0(sg, a)
                assert list(tiles[b:b + lv, c]) == f, (t, c, a)


def test_coverage_and_uniformity():
    # a space of 18 x 6 x 3 schedules per axis triple: every schedule of every axis appears, at about its share
    sg = w.gemm(12, 4, 4, hw=w.toy_device(), rd_levels=2)
    n = 60000
    seg, tiles = _generate([sg], [n], seed=5)
    for a in range(3):
        lv, b = _levels(sg, a), _slot0(sg, a)
        space = _factorisations(sg.extent[a], lv)
        seen, counts = np.unique(tiles[b:b + lv].T, axis=0, return_counts=True)
        assert sorted(map(tuple, seen.tolist())) == sorted(space)
        expect = n / len(space)
        chi2 = float(((counts - expect) ** 2 / expect).sum())
        assert chi2 < 3.0 * len(space) + 30                                  # dof = len(space) - 1; far above any plausible draw
    # axes are independent: the pair (axis 0 schedule, axis 1 schedule) covers the product space
    pairs = np.unique(tiles[0:8].T, axis=0)
    assert len(pairs) == len(_factorisations(12, 4)) * len(_factorisations(4, 4))


def test_schedule_depends_on_global_index_and_seed_only():
    sg = SGS[0]
    seg1, one = _generate([sg], [200], seed=9)
    seg2, two = _generate([sg, sg], [120, 80], seed=9)
    assert (one == two).all()
    _, other = _generate([sg], [200], seed=10)
    assert (one != other).any()
    assert len(np.unique(one.T, axis=0)) > 150                              # candidates differ from each other


def test_fragment_must_divide_the_extent():
    bad = w.gemm(64, 72, 64, dtype_bytes=2, hw=w.toy_device(), rd_levels=3, frag=(16, 16, 16))
    with pytest.raises(oracle.OracleError):
        oracle.random_init([bad], np.array([0, 4]), w.n_slots(bad), 1)
