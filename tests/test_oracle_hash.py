"""Pins for the oracle's cross-polytope hash (Section 3.2, Eq. 3).

None of these re-types the oracle's formula: they use the geometric
definition (nearest vertex of the cross-polytope by Euclidean distance),
pure-Python exact integer arithmetic, invariants and hand-worked cases.
"""
import os

import numpy as np
import pytest

from oracle import hash_ref, combine_codes, widen
from workloads import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


# ---------------------------------------------------------------- C1 brute force
def _nearest_vertex_code(y):
    """Geometric definition: among the 2r vertices +-e_i pick the one closest
    to y in squared Euclidean distance.  Equidistant vertices are resolved
    towards the lowest coordinate index, then towards the positive vertex
    (visiting order +e_0, -e_0, +e_1, -e_1, ...).  Vertex +e_i is numbered i,
    -e_i is numbered i + r.  Pure Python, exact for integer y."""
    r = len(y)
    best, best_d = None, None
    for i in range(r):
        for s in (1, -1):
            dist = sum((y[j] - (s if j == i else 0)) ** 2 for j in range(r))
            if best_d is None or dist < best_d:
                best, best_d = (i if s > 0 else i + r), dist
    return best


def _brute_hash(x_rows, R):
    L, r, d = len(R), len(R[0]), len(R[0][0])
    buckets, codes = [], []
    for x in x_rows:
        cs = []
        for l in range(L):
            y = [sum(R[l][i][j] * x[j] for j in range(d)) for i in range(r)]
            cs.append(_nearest_vertex_code(y))
        b = 0
        for c in cs:
            b = b * (2 * r) + c
        buckets.append(b)
        codes.append(cs)
    return buckets, codes


@pytest.mark.parametrize("seed,T,d,L,r", [(0, 64, 16, 2, 4), (1, 48, 8, 3, 8), (2, 33, 5, 1, 3), (3, 20, 12, 4, 2)])
def test_hash_matches_nearest_vertex_brute_force(seed, T, d, L, r):
    rng = np.random.default_rng(seed)
    # small integers: every product and sum is exact in any order, so the
    # comparison is bit-exact and ties (there are many) exercise the tie rule
    x = rng.integers(-6, 7, size=(T, d))
    R = rng.integers(-5, 6, size=(L, r, d))
    bucket, code, margin, runner = hash_ref(_f32(x), _f32(R), "f32")
    bb, cc = _brute_hash(x.tolist(), R.tolist())
    assert code.tolist() == cc
    assert [int(b) for b in bucket] == bb


def test_distance_to_vertex_is_minimal_random_float():
    # float data: the chosen vertex must be a nearest one (distance check, not argmax)
    rng = np.random.default_rng(7)
    T, d, L, r = 200, 24, 2, 8
    x = _f32(rng.standard_normal((T, d)))
    R = _f32(rng.standard_normal((L, r, d)))
    _, code, _, _ = hash_ref(x, R, "f32")
    for l in range(L):
        y = x.astype(np.float64) @ R[l].astype(np.float64).T
        verts = np.concatenate([np.eye(r), -np.eye(r)])          # [2r, r]
        dist = ((y[:, None, :] - verts[None]) ** 2).sum(-1)      # [T, 2r]
        chosen = dist[np.arange(T), code[:, l]]
        assert np.all(chosen <= dist.min(axis=1) + 1e-12)


# ---------------------------------------------------------------- C2 invariants
def _rand_case(seed, T=300, d=32, L=3, r=8, dtype="f32"):
    rng = np.random.default_rng(seed)
    x = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    R = synth.f32_to_storage(rng.standard_normal((L, r, d)).astype(np.float32), dtype)
    return x, R


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("p", [-3, 1, 5])
def test_positive_scaling_invariance(dtype, p):
    x, R = _rand_case(11, dtype=dtype)
    xs = synth.f32_to_storage(synth.storage_to_f32(x, dtype) * np.float32(2.0 ** p), dtype)  # exact
    b0, c0, m0, _ = hash_ref(x, R, dtype)
    b1, c1, m1, _ = hash_ref(xs, R, dtype)
    assert np.array_equal(b0, b1) and np.array_equal(c0, c1)
    assert np.allclose(m0, m1, rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_negation_flips_sign_only(dtype):
    x, R = _rand_case(12, dtype=dtype)
    L, r, _ = R.shape
    xn = synth.f32_to_storage(-synth.storage_to_f32(x, dtype), dtype)
    _, c0, _, _ = hash_ref(x, R, dtype)
    _, c1, _, _ = hash_ref(xn, R, dtype)
    assert np.array_equal(c0 % r, c1 % r)                 # same coordinate
    assert np.array_equal((c0 // r) ^ 1, c1 // r)         # opposite vertex
    assert c0.min() >= 0 and c0.max() < 2 * r


def test_row_permutation_of_R_permutes_codes():
    x, R = _rand_case(13)
    L, r, _ = R.shape
    rng = np.random.default_rng(5)
    _, c0, _, _ = hash_ref(x, R, "f32")
    for l in range(L):
        pi = rng.permutation(r)                           # new row j = old row pi[j]
        Rp = R.copy()
        Rp[l] = R[l][pi]
        _, c1, _, _ = hash_ref(x, Rp, "f32")
        inv = np.argsort(pi)
        expect = c0.copy()
        expect[:, l] = inv[c0[:, l] % r] + r * (c0[:, l] // r)
        assert np.array_equal(c1, expect)


def test_each_hash_uses_its_own_rotation_and_digit_order():
    # swapping two rotations swaps the two digits; hash 0 is the most significant
    x, R = _rand_case(14, L=2, r=8)
    b0, c0, _, _ = hash_ref(x, R, "f32")
    b1, c1, _, _ = hash_ref(x, R[::-1].copy(), "f32")
    assert np.array_equal(c0[:, 0], c1[:, 1]) and np.array_equal(c0[:, 1], c1[:, 0])
    assert np.array_equal(b0, c0[:, 0].astype(np.uint64) * 16 + c0[:, 1].astype(np.uint64))


# ---------------------------------------------------------------- C3 closed forms
def test_identity_rows_give_signed_argmax_of_leading_coordinates():
    # fixture: hand-worked, see the file's header
    rows = []
    with open(os.path.join(GOLDEN, "hash_identity_cases.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            vec, code = line.split("->")
            rows.append(([float(v) for v in vec.split()], int(code)))
    d, r = 6, 4
    R = np.zeros((1, r, d), np.float32)
    R[0, np.arange(r), np.arange(r)] = 1.0
    x = _f32([v for v, _ in rows])
    bucket, code, _, _ = hash_ref(x, R, "f32")
    assert code[:, 0].tolist() == [c for _, c in rows]
    assert bucket.tolist() == [c for _, c in rows]


def test_orthonormal_rows_hash_their_own_directions():
    rng = np.random.default_rng(21)
    d, r, L = 24, 8, 2
    R = np.empty((L, r, d), np.float32)
    for l in range(L):
        q, _ = np.linalg.qr(rng.standard_normal((d, d)))
        R[l] = q[:, :r].T.astype(np.float32)
    for l in range(L):
        for i in range(r):
            for s in (1.0, -1.0):
                x = _f32(s * 3.0 * R[l, i][None, :])
                _, code, margin, _ = hash_ref(x, R, "f32")
                assert code[0, l] == i + (r if s < 0 else 0)
                assert margin[0, l] > 0.999          # every other coordinate is ~0


def test_mixed_radix_combination_by_hand():
    # digits (3, 0, 7) in base 8 = 3*64 + 0*8 + 7; digits (1, 9) in base 10 = 19
    assert combine_codes(np.array([[3, 0, 7]], np.int32), 4).tolist() == [3 * 64 + 7]
    assert combine_codes(np.array([[1, 9], [9, 1]], np.int32), 5).tolist() == [19, 91]
    # largest supported: (2r)^L just below 2^63 keeps every digit
    L, r = 9, 64
    code = np.full((1, L), 2 * r - 1, np.int32)
    assert int(combine_codes(code, r)[0]) == (2 * r) ** L - 1


# ---------------------------------------------------------------- tie rule / margin
def test_tie_rule_and_zero_token():
    R = np.zeros((1, 4, 4), np.float32)
    R[0] = np.eye(4)
    x = _f32([[0, 0, 0, 0],          # zero token: code 0, margin 0
              [2, -2, 2, 1],         # |.| tie between 0,1,2 -> lowest index, positive
              [-2, 2, 0, 0],         # tie 0,1 -> index 0, negative -> 0 + r
              [1, 3, -4, 2]])        # clear winner: index 2 negative; runner-up index 1 positive
    _, code, margin, runner = hash_ref(x, R, "f32")
    assert code[:, 0].tolist() == [0, 0, 4, 6]
    assert margin[0, 0] == 0.0 and margin[1, 0] == 0.0 and margin[2, 0] == 0.0
    assert margin[3, 0] == pytest.approx(0.25)
    assert runner[3, 0] == 1
    assert runner[2, 0] == 1          # the other tied coordinate (positive)


def test_margin_and_runner_up_definition():
    x, R = _rand_case(15, T=100, d=16, L=2, r=6)
    _, code, margin, runner = hash_ref(x, R, "f32")
    r = R.shape[1]
    for l in range(2):
        y = widen(x, "f32") @ widen(R[l], "f32").T
        for t in range(100):
            order = sorted(range(r), key=lambda i: (-abs(y[t, i]), i))
            m1, m2 = abs(y[t, order[0]]), abs(y[t, order[1]])
            assert margin[t, l] == pytest.approx((m1 - m2) / m1, abs=1e-15)
            assert runner[t, l] % r == order[1]
            assert (runner[t, l] >= r) == (y[t, order[1]] < 0)


# ---------------------------------------------------------------- C5 locality
def test_closer_pairs_collide_at_least_as_often():
    # LSH property (Section 2.3): collision probability does not increase with angle
    rng = np.random.default_rng(31)
    d, r, L, n = 32, 8, 1, 4000
    R = _f32(rng.standard_normal((L, r, d)))
    base = rng.standard_normal((n, d))
    base /= np.linalg.norm(base, axis=1, keepdims=True)
    other = rng.standard_normal((n, d))
    other -= (other * base).sum(1, keepdims=True) * base
    other /= np.linalg.norm(other, axis=1, keepdims=True)
    rates = []
    for angle in (0.05, 0.3, 0.8, 1.4):
        y = np.cos(angle) * base + np.sin(angle) * other
        b0, _, _, _ = hash_ref(_f32(base), R, "f32")
        b1, _, _, _ = hash_ref(_f32(y), R, "f32")
        rates.append(float((b0 == b1).mean()))
    assert rates[0] > 0.85
    assert all(rates[i] >= rates[i + 1] - 0.02 for i in range(3))
    assert rates[-1] < rates[0] - 0.3


def test_bf16_inputs_are_widened_exactly():
    # the same values stored as bf16 or as fp32 hash identically
    x, R = _rand_case(16, dtype="bf16")
    x32, R32 = synth.storage_to_f32(x, "bf16"), synth.storage_to_f32(R, "bf16")
    a = hash_ref(x, R, "bf16")
    b = hash_ref(x32, R32, "f32")
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_gate_logits_against_python_loops_and_unit_vectors():
    # E != d and T != E, so a transposed operand cannot pass
    from oracle import gate_logits_ref, widen
    rng = np.random.default_rng(11)
    T, d, E = 7, 12, 5
    for dtype in ("f32", "bf16"):
        x = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
        w = synth.f32_to_storage(rng.standard_normal((E, d)).astype(np.float32), dtype)
        got = gate_logits_ref(x, w, dtype)
        assert got.shape == (T, E) and got.dtype == np.float64
        x64, w64 = widen(x, dtype), widen(w, dtype)
        for t in range(T):
            for e in range(E):
                assert abs(got[t, e] - sum(float(x64[t, i]) * float(w64[e, i]) for i in range(d))) < 1e-12
        unit = np.zeros((E, d), np.float32)
        unit[np.arange(E), [3, 0, 11, 7, 5]] = 1.0          # gate row e picks out one coordinate
        assert np.array_equal(gate_logits_ref(x, synth.f32_to_storage(unit, dtype), dtype), x64[:, [3, 0, 11, 7, 5]])
