"""The seeded input generators: counts, determinism, structure."""
import numpy as np

import workloads as w


def test_ordered_factorisation_counts_match_the_closed_form():
    # prod over prime powers p^e of C(e + L - 1, L - 1)
    for n, L, want in ((512, 4, 220), (512, 2, 10), (768, 4, 660), (3072, 4, 1144), (56, 4, 80), (64, 4, 84),
                       (4096, 4, 455), (256, 4, 165), (28, 4, 40), (1, 4, 1), (7, 3, 3)):
        t = w.ordered_factorizations(n, L)
        assert len(t) == want == w.count_ordered_factorizations(n, L)
        assert np.all(np.prod(t.astype(np.int64), axis=1) == n)
        assert len({tuple(r) for r in t}) == len(t)
        assert [tuple(r) for r in t] == sorted(tuple(r) for r in t)   # lexicographic


def test_populations_are_reproducible_and_sliceable():
    sg = w.conv2d(1, 64, 56, 56, 64, 3, 3)
    a, aa = w.sample_population(sg, 1000, seed=7, stream=3)
    b, ba = w.sample_population(sg, 1000, seed=7, stream=3)
    c, ca = w.sample_population(sg, 100, seed=7, stream=3, first=400)
    assert np.array_equal(a, b) and np.array_equal(aa, ba)
    assert np.array_equal(a[:, 400:500], c) and np.array_equal(aa[400:500], ca)
    d, _ = w.sample_population(sg, 1000, seed=8, stream=3)
    assert not np.array_equal(a, d)
    assert a.shape == (22, 1000) and a.dtype == np.uint16
    slot = 0
    for axis, ext in enumerate(sg.extent):
        L = 4 if axis < 4 else 2
        assert np.all(np.prod(a[slot:slot + L].astype(np.int64), axis=0) == ext)
        slot += L
    assert set(np.unique(aa & 0xFF)) <= {0, 1, 2, 3} and set(np.unique(aa >> 8)) <= {0, 1, 2}


def test_fragment_constraint_on_inner_tiles():
    sg = w.gemm(4096, 4096, 4096, dtype_bytes=2, rd_levels=3, frag=(16, 16, 16))
    t, _ = w.sample_population(sg, 5000, seed=0)
    assert t.shape == (11, 5000)
    assert np.all(t[3] % 16 == 0) and np.all(t[7] % 16 == 0) and np.all(t[10] % 16 == 0)
    assert np.all(np.prod(t[8:11].astype(np.int64), axis=0) == 4096)


def test_config_shapes():
    c0 = w.make_config(0)
    assert c0.n == 4096 and c0.k_draft == 64 and c0.tiles.shape == (10, 4096)
    c1 = w.make_config(1, scale=1 / 64)
    assert c1.n == 1024 and c1.tiles.shape[0] == 22
    c3 = w.make_config(3, scale=0.02)
    assert len(c3.subgraphs) == 20 and c3.n == 20 * 1000 and c3.tiles.shape[0] == 14 and c3.k_final == 32
    assert [sg.n_sp for sg in c3.subgraphs[:6]] == [2, 3, 3, 2, 2, 2]
    assert np.all(c3.tiles[10:, c3.seg_off[0]:c3.seg_off[1]] == 0)     # unused slots of a 10-slot subgraph
    c4 = w.make_config(4, scale=1 / 4096)
    assert c4.n == 4096 + 1024 and c4.tiles.shape[0] == 20


def test_bf16_bit_helpers_and_features():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 0.0], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert list(w.bf16_bits_to_f32(w.f32_to_bf16_bits(x))[:3]) == [1.0, 1.0, 1.015625]
    f = w.make_statement_features(np.array([5, 9, 5]), [3, 8, 3])
    assert f.shape == (3, 8, 164) and np.array_equal(f[0], f[2]) and not np.array_equal(f[0], f[1])
    assert np.all(f[0, 3:] == 0) and f.min() >= 0 and f.max() < 24
    assert 0.4 < (f[1] == 0).mean() < 0.6
    m = w.make_mlp_weights(seed=1)
    assert m["W1"].shape == (256, 164) and m["W2"].shape == (256, 256) and m["w3"].shape == (256,)
    assert np.abs(w.bf16_bits_to_f32(m["W1"])).max() <= 1 / np.sqrt(164) * 1.01
