"""Pins for the oracle's spherical hash (the "SP" family of the ablation in Section 4.5).  The paper names the
family without defining it, so these pins tie the oracle to the reading it states - bit l is 1 inside or on the
sphere (pivot l, squared radius l) - and to what that definition implies; parity with the paper itself is unpinned."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import sphere_hash_ref, narrow, widen
from workloads import synth


def test_brute_force_in_exact_integer_arithmetic():
    # small integers: squared distances are exact integers, many tokens sit exactly on a sphere
    rng = np.random.default_rng(0)
    T, d, B = 200, 5, 7
    x = rng.integers(-4, 5, size=(T, d)).astype(np.float32)
    p = rng.integers(-3, 4, size=(B, d)).astype(np.float32)
    t2 = rng.integers(0, 60, size=B).astype(np.float64)
    bucket, bit, margin = sphere_hash_ref(x, p, t2, "f32")
    on_surface = 0
    for t in range(T):
        code = 0
        for l in range(B):
            dist2 = sum((int(x[t, i]) - int(p[l, i])) ** 2 for i in range(d))
            inside = dist2 <= int(t2[l])
            on_surface += dist2 == int(t2[l])
            assert bit[t, l] == inside
            assert (margin[t, l] == 0.0) == (dist2 == int(t2[l]))
            code = code * 2 + int(inside)
        assert int(bucket[t]) == code
    assert on_surface > 5        # the "on the sphere counts as inside" rule was exercised


def test_bit_order_and_radius_by_hand():
    # one token at the origin; pivots at distance 1, 2, 3 along an axis; squared radii 1, 3.9, 9
    #   bit 0: 1 <= 1 -> 1 (on the sphere); bit 1: 4 <= 3.9 -> 0; bit 2: 9 <= 9 -> 1   => code 0b101 = 5
    x = np.zeros((1, 3), np.float32)
    p = np.array([[1, 0, 0], [0, 2, 0], [0, 0, -3]], np.float32)
    bucket, bit, margin = sphere_hash_ref(x, p, np.array([1.0, 3.9, 9.0]), "f32")
    assert bit.tolist() == [[1, 0, 1]] and int(bucket[0]) == 5
    assert margin[0, 0] == 0.0 and abs(margin[0, 1] - 0.1 / 4.0) < 1e-15 and margin[0, 2] == 0.0
    # a single sphere: the code is the bit
    b1, _, _ = sphere_hash_ref(x, p[:1], np.array([0.5]), "f32")
    assert int(b1[0]) == 0


def test_translation_invariance_and_radius_monotonicity():
    rng = np.random.default_rng(1)
    T, d, B = 300, 8, 10
    x = rng.integers(-8, 9, size=(T, d)).astype(np.float32)
    p = rng.integers(-8, 9, size=(B, d)).astype(np.float32)
    t2 = rng.integers(50, 300, size=B).astype(np.float64)
    v = rng.integers(-5, 6, size=d).astype(np.float32)
    b0, bit0, _ = sphere_hash_ref(x, p, t2, "f32")
    b1, _, _ = sphere_hash_ref(x + v, p + v, t2, "f32")            # moving tokens and pivots together changes nothing
    assert np.array_equal(b0, b1)
    _, bit_big, _ = sphere_hash_ref(x, p, t2 + 40.0, "f32")           # a larger sphere keeps every inside token inside
    assert np.all(bit_big >= bit0) and (bit_big > bit0).any()
    _, none, _ = sphere_hash_ref(x, p, np.full(B, -1.0), "f32")       # negative squared radius: nothing is inside
    assert not none.any()
    _, every, _ = sphere_hash_ref(x, p, np.full(B, 1e9), "f32")
    assert every.all()


def test_far_pivots_give_hyperplane_hashing():
    # pivot p = -s a (|a| = 1) with squared radius (s + b)^2: for s -> infinity the sphere's surface near the
    # origin is the plane <a, x> = b, and the bit is [<a, x> <= b]
    rng = np.random.default_rng(2)
    T, d, B = 500, 6, 8
    x = rng.standard_normal((T, d))
    a = rng.standard_normal((B, d))
    a /= np.linalg.norm(a, axis=1, keepdims=True)
    b = rng.standard_normal(B) * 0.3
    s = 1e7
    _, bit, _ = sphere_hash_ref(x, -s * a, (s + b) ** 2, "f64")
    plane = (x @ a.T) <= b
    # ||x + s a||^2 = s^2 + 2 s <a, x> + |x|^2, so the two differ only where |<a, x> - b| < |x|^2 / (2 s) ~ 1e-6
    clear = np.abs(x @ a.T - b) > 1e-5
    assert clear.mean() > 0.99
    assert np.array_equal(bit.astype(bool)[clear], plane[clear])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_storage_types_are_widened_exactly(dtype):
    rng = np.random.default_rng(3)
    T, d, B = 100, 16, 12
    x = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    p = synth.f32_to_storage(rng.standard_normal((B, d)).astype(np.float32), dtype)
    t2 = np.full(B, 2.0 * d)
    b_s, bit_s, m_s = sphere_hash_ref(x, p, t2, dtype)
    b_w, bit_w, m_w = sphere_hash_ref(widen(x, dtype), widen(p, dtype), t2, "f64")
    assert np.array_equal(b_s, b_w) and np.array_equal(bit_s, bit_w) and np.array_equal(m_s, m_w)
    # exact rational check of one token against one sphere
    xe = [Fraction(float(v)) for v in widen(x, dtype)[0]]
    pe = [Fraction(float(v)) for v in widen(p, dtype)[0]]
    assert bit_s[0, 0] == (sum((u - v) ** 2 for u, v in zip(xe, pe)) <= Fraction(2 * d))
    assert 0.2 < bit_s.mean() < 0.8       # radius^2 = 2 d is the mean squared distance of two unit Gaussians: balanced bits
