"""Pins of the oracle's momentum online adaptation step (Sec. 4.3, Update_MoA of Alg. 1, m = 0.99).

The update's formula sits in a lost figure; the reading (momentum-contrast form, phi_s <- m phi_s + (1 - m) phi_t) is
"parity unpinned" by the paper.  Pinned here: the special cases, the closed form of repeated updates, the equivalence
with the gradient form, and the bfloat16 copy.
"""
import numpy as np
import pytest

import oracle
import workloads as w


def _params(n, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(-0.1, 0.1, n).astype(np.float32), rng.uniform(-0.1, 0.1, n).astype(np.float32)


def test_special_cases():
    s, t = _params(1000, 1)
    assert np.array_equal(oracle.moa_update(s, t, 1.0)[0], s)          # m = 1: the Siamese model never moves
    assert np.array_equal(oracle.moa_update(s, t, 0.0)[0], t)          # m = 0: it is the target model
    new, _, f64 = oracle.moa_update(s, s, 0.99)                        # target unchanged: a fixed point up to rounding
    assert np.abs(new - s).max() <= 2 * np.spacing(np.abs(s).max())
    assert np.allclose(f64, s, rtol=1e-7, atol=0)


def test_hand_values():
    # exactly representable: m = 0.5
    new, bf, f64 = oracle.moa_update(np.array([1.0, -2.0, 0.25], np.float32), np.array([3.0, 2.0, 0.75], np.float32), 0.5)
    assert list(new) == [2.0, 0.0, 0.5] and list(f64) == [2.0, 0.0, 0.5]
    assert list(bf) == [0x4000, 0x0000, 0x3F00]
    # m = 0.99 as binary32, each operation rounded separately
    m = np.float32(0.99)
    c = np.float32(1.0) - m
    s, t = np.float32(0.3), np.float32(-0.7)
    want = np.float32(np.float32(m * s) + np.float32(c * t))
    assert oracle.moa_update([s], [t], m)[0][0] == want


def test_repeated_updates_follow_the_closed_form():
    # with a fixed target, r updates leave phi_s - phi_t = m^r (phi_s(0) - phi_t)
    s0, t = _params(500, 2)
    s, m, r = s0.copy(), 0.99, 300
    for _ in range(r):
        s = oracle.moa_update(s, t, m)[0]
    want = t.astype(np.float64) + (float(np.float32(m)) ** r) * (s0.astype(np.float64) - t.astype(np.float64))
    assert np.abs(s - want).max() <= 300 * 2 * np.spacing(np.float32(0.2))


def test_equals_the_gradient_form():
    # phi_t = phi_s - lr * g  =>  m phi_s + (1 - m) phi_t = phi_s - (1 - m) lr g
    rng = np.random.default_rng(3)
    s = rng.uniform(-0.1, 0.1, 2000).astype(np.float32)
    g = rng.normal(0, 1, 2000).astype(np.float32)
    lr = 1e-3
    t = (s.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
    _, _, f64 = oracle.moa_update(s, t, 0.99)
    want = s.astype(np.float64) - (1.0 - float(np.float32(0.99))) * (s.astype(np.float64) - t.astype(np.float64))
    assert np.allclose(f64, want, rtol=0, atol=1e-12)
    new = oracle.moa_update(s, t, 0.99)[0]
    assert np.abs(new - f64).max() <= 2 * np.spacing(np.float32(0.1))


def test_bfloat16_copy_rounds_to_nearest_even():
    s = np.array([1.00390625, 1.01171875, -1.00390625, 3.0e-39], np.float32)    # two ties, a negative tie, a subnormal
    new, bf, _ = oracle.moa_update(s, s, 1.0)
    assert np.array_equal(new, s)
    assert list(bf[:3]) == [0x3F80, 0x3F82, 0xBF80]
    assert np.array_equal(bf, w.f32_to_bf16_bits(new))                          # the workloads' packer: an independent routine


def test_bad_arguments():
    with pytest.raises(oracle.OracleError):
        oracle.moa_update([0.0], [0.0], 1.5)
    with pytest.raises(oracle.OracleError):
        oracle.moa_update([0.0], [0.0], float("nan"))
