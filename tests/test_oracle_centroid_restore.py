"""Pins for the oracle's centroid (Section 2.3 centroid formula, Alg. 1 "Mean")
and restore (Eq. 4, Eq. 5) steps, and for its storage rounding."""
import numpy as np
import pytest
import torch

from oracle import group_ref, centroid_ref, restore_ref, widen, narrow
from workloads import synth


def _case(seed, T=400, d=24, k=2, E=6, nb=30, dtype="f32"):
    rng = np.random.default_rng(seed)
    x = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    expert = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    bucket = rng.integers(0, nb, size=T).astype(np.uint64)
    return x, expert, bucket, group_ref(expert, bucket, E)


# ------------------------------------------------------------------ rounding
def test_narrow_bf16_matches_torch_and_hand_cases():
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000),
                        [0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                         3.3895313892515355e38]])
    got = narrow(v, "bf16")
    ref = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1; 1 + 3*2^-8 -> 1 + 2^-6
    assert widen(narrow(np.array([1.0 + 2.0 ** -8]), "bf16"), "bf16")[0] == 1.0
    assert widen(narrow(np.array([1.0 + 3 * 2.0 ** -8]), "bf16"), "bf16")[0] == 1.0 + 2.0 ** -6
    assert widen(narrow(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]), "bf16"), "bf16")[0] == 1.0 + 2.0 ** -7


def test_widen_narrow_round_trip_is_identity():
    bits = np.arange(0, 0x7F80, dtype=np.uint16)                  # every finite non-negative bf16
    assert np.array_equal(narrow(widen(bits, "bf16"), "bf16"), bits)
    f = np.random.default_rng(1).standard_normal(1000).astype(np.float32)
    assert np.array_equal(narrow(widen(f, "f32"), "f32"), f)


# ------------------------------------------------------------------ centroid
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_centroid_python_loop_and_mass_conservation(dtype):
    x, expert, bucket, g = _case(3, dtype=dtype)
    k = expert.shape[1]
    c, c64 = centroid_ref(x, g["perm"], g["seg_offsets"], k, dtype, return_f64=True)
    x64 = widen(x, dtype)
    # plain loop over clusters, members summed one at a time
    for s in range(g["S"]):
        acc = np.zeros(x.shape[1])
        members = g["perm"][g["seg_offsets"][s]:g["seg_offsets"][s + 1]]
        for a in members:
            acc += x64[a // k]
        assert np.allclose(c64[s], acc / len(members), rtol=1e-15, atol=1e-15)
    # mass conservation per expert: sum_s n_s c_s == sum of the expert's token rows
    n = np.diff(g["seg_offsets"]).astype(np.float64)
    for e in range(6):
        lo, hi = g["expert_offsets"][e], g["expert_offsets"][e + 1]
        lhs = (n[lo:hi, None] * c64[lo:hi]).sum(0)
        rhs = x64[np.nonzero(expert == e)[0]].sum(0)
        assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    assert np.array_equal(c, narrow(c64, dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_centroid_matches_torch_index_add(dtype):
    x, expert, bucket, g = _case(4, T=1000, d=16, dtype=dtype)
    k = expert.shape[1]
    _, c64 = centroid_ref(x, g["perm"], g["seg_offsets"], k, dtype, return_f64=True)
    xt = torch.from_numpy(widen(x, dtype))
    acc = torch.zeros(g["S"], x.shape[1], dtype=torch.float64)
    acc.index_add_(0, torch.from_numpy(g["seg_of"].astype(np.int64)), xt[torch.arange(expert.size) // k])
    cnt = torch.bincount(torch.from_numpy(g["seg_of"].astype(np.int64)), minlength=g["S"]).to(torch.float64)
    assert np.allclose(c64, (acc / cnt[:, None]).numpy(), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_singleton_and_identical_member_centroids_are_exact(dtype):
    rng = np.random.default_rng(5)
    T, d = 60, 8
    x = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    x[10:20] = x[10]                                   # ten identical tokens
    expert = np.zeros((T, 1), np.int32)
    bucket = np.arange(T).astype(np.uint64)
    bucket[10:20] = 10                                 # ... in one bucket
    g = group_ref(expert, bucket, 1)
    c = centroid_ref(x, g["perm"], g["seg_offsets"], 1, dtype)
    toks = g["perm"][g["seg_offsets"][:-1]]
    assert np.array_equal(c, x[toks])                  # bit-exact in storage form


# ------------------------------------------------------------------ restore
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_token_its_own_bucket_reconstructs_exactly(dtype):
    rng = np.random.default_rng(6)
    T, d, k, E = 200, 16, 2, 4
    x = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    expert = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    bucket = rng.permutation(T).astype(np.uint64)
    g = group_ref(expert, bucket, E)
    assert g["S"] == T * k
    c = centroid_ref(x, g["perm"], g["seg_offsets"], k, dtype)
    ec = synth.f32_to_storage(rng.standard_normal((g["S"], d)).astype(np.float32), dtype)
    y = restore_ref(x, c, ec, g["seg_of"], k, dtype)
    assert np.array_equal(y, ec[g["seg_of"]])          # Y = E(x) bit for bit


@pytest.mark.parametrize("dtype,tol", [("f32", 2.0 ** -23), ("bf16", 2.0 ** -7)])
def test_identity_expert_returns_the_token(dtype, tol):
    x, expert, bucket, g = _case(7, dtype=dtype)
    k = expert.shape[1]
    c = centroid_ref(x, g["perm"], g["seg_offsets"], k, dtype)
    y = restore_ref(x, c, c, g["seg_of"], k, dtype)    # E = identity: E(c) = c
    x64 = widen(x, dtype)[np.arange(expert.size) // k]
    y64 = widen(y, dtype)
    # c + (x - c) in binary64 is x up to one rounding of the sum, then one storage rounding
    assert np.all(np.abs(y64 - x64) <= tol * np.maximum(np.abs(x64), np.abs(widen(c, dtype)[g["seg_of"]])) + 1e-30)


def test_segment_sum_invariant_and_linear_expert_closed_form():
    # E(x) = W x.  Then Y_a - W x_a = (I - W)(x_a - c_s), and sum over a cluster of Y_a = n_s E(c_s)
    rng = np.random.default_rng(8)
    x, expert, bucket, g = _case(8, T=300, d=12, k=1, E=3, nb=10)
    d = x.shape[1]
    W = rng.standard_normal((d, d)) / np.sqrt(d)
    c = centroid_ref(x, g["perm"], g["seg_offsets"], 1, "f32")
    c64 = widen(c, "f32")
    ec = narrow(c64 @ W.T, "f32")
    y64 = widen(restore_ref(x, c, ec, g["seg_of"], 1, "f32"), "f32")
    x64 = widen(x, "f32")
    s = g["seg_of"]
    lhs = y64 - x64 @ W.T
    rhs = (x64 - c64[s]) @ (np.eye(d) - W).T
    assert np.allclose(lhs, rhs, rtol=0, atol=2e-6)
    n = np.diff(g["seg_offsets"])
    ysum = np.zeros_like(c64)
    np.add.at(ysum, s, y64)
    assert np.allclose(ysum, n[:, None] * widen(ec, "f32"), rtol=0, atol=1e-5 * n.max())


def test_residual_sign_and_no_residual_flag():
    # one cluster of two tokens, by hand: c = (x0 + x1)/2; Y0 = EC + (x0 - c)
    x = np.array([[1.0, 4.0], [3.0, 0.0]], np.float32)
    g = group_ref(np.zeros((2, 1), np.int32), np.zeros(2, np.uint64), 1)
    c = centroid_ref(x, g["perm"], g["seg_offsets"], 1, "f32")
    assert c.tolist() == [[2.0, 2.0]]
    ec = np.array([[10.0, 20.0]], np.float32)
    y = restore_ref(x, c, ec, g["seg_of"], 1, "f32")
    assert y.tolist() == [[9.0, 22.0], [11.0, 18.0]]
    y0 = restore_ref(x, c, ec, g["seg_of"], 1, "f32", no_residual=True)
    assert y0.tolist() == [[10.0, 20.0], [10.0, 20.0]]


def test_gate_weighted_combine_by_hand():
    # token 0 goes to experts (0, 1) with weights (0.25, 0.75): out = 0.25*Y[0] + 0.75*Y[1]
    x = np.array([[2.0, 2.0]], np.float32)
    expert = np.array([[0, 1]], np.int32)
    g = group_ref(expert, np.zeros(1, np.uint64), 2)
    c = centroid_ref(x, g["perm"], g["seg_offsets"], 2, "f32")
    ec = np.array([[4.0, 8.0], [12.0, 16.0]], np.float32)
    w = np.array([[0.25, 0.75]], np.float32)
    y = restore_ref(x, c, ec, g["seg_of"], 2, "f32", gate_weight=w)
    assert y.tolist() == [[10.0, 14.0]]


def test_gate_weighted_combine_two_tokens_shared_cluster_by_hand():
    # Two tokens, both routed to experts (0, 1), both in bucket 0: clusters {a0, a2} (expert 0) and {a1, a3}
    # (expert 1), each with centroid c = (x0 + x1)/2 = (2, 5) and non-zero residuals -+(1, 2).
    #   Y[a0] = EC0 + (x0 - c) = (10, 20) + (-1, 2) = ( 9, 22)     Y[a1] = EC1 + (x0 - c) = (100, 200) + (-1, 2) = ( 99, 202)
    #   Y[a2] = EC0 + (x1 - c) = (11, 18)                          Y[a3] = EC1 + (x1 - c) = (101, 198)
    #   out[0] = 0.25*Y[a0] + 0.5*Y[a1] = (2.25 + 49.5, 5.5 + 101) = (51.75, 106.5)     (weights need not sum to 1)
    #   out[1] = 2*Y[a2] - 1*Y[a3]      = (22 - 101, 36 - 198)     = (-79, -162)
    x = np.array([[1.0, 7.0], [3.0, 3.0]], np.float32)
    expert = np.array([[0, 1], [0, 1]], np.int32)
    g = group_ref(expert, np.zeros(2, np.uint64), 2)
    assert g["seg_of"].tolist() == [0, 1, 0, 1]
    c = centroid_ref(x, g["perm"], g["seg_offsets"], 2, "f32")
    assert c.tolist() == [[2.0, 5.0], [2.0, 5.0]]
    ec = np.array([[10.0, 20.0], [100.0, 200.0]], np.float32)
    w = np.array([[0.25, 0.5], [2.0, -1.0]], np.float32)
    out = restore_ref(x, c, ec, g["seg_of"], 2, "f32", gate_weight=w)
    assert out.shape == (2, 2)
    assert out.tolist() == [[51.75, 106.5], [-79.0, -162.0]]
    # without the residual only the expert outputs are mixed
    out0 = restore_ref(x, c, ec, g["seg_of"], 2, "f32", no_residual=True, gate_weight=w)
    assert out0.tolist() == [[52.5, 105.0], [-80.0, -160.0]]


@pytest.mark.parametrize("k", [2, 3])
def test_gate_weighted_combine_is_the_weighted_sum_of_the_unweighted_rows(k):
    # Eq. 2 over Eq. 4/5: restore_ref(gate_weight=w)[t] == sum_j w[t, j] * restore_ref(...)[t*k + j], nothing rounded
    x, expert, bucket, g = _case(21 + k, T=300, d=10, k=k, E=5, nb=12, dtype="f32")
    rng = np.random.default_rng(99)
    x64 = widen(x, "f32")
    _, c64 = centroid_ref(x, g["perm"], g["seg_offsets"], k, "f32", return_f64=True)
    assert (np.diff(g["seg_offsets"]) > 1).sum() > 20            # residuals are not all zero
    ec64 = rng.standard_normal((g["S"], x.shape[1]))
    w = rng.standard_normal((x.shape[0], k))
    y = restore_ref(x64, c64, ec64, g["seg_of"], k, "f64")        # [N, d]
    assert np.abs(y - ec64[g["seg_of"]]).max() > 0.1
    out = restore_ref(x64, c64, ec64, g["seg_of"], k, "f64", gate_weight=w)
    ref = np.zeros((x.shape[0], x.shape[1]))
    for t in range(x.shape[0]):
        for j in range(k):
            ref[t] += w[t, j] * y[t * k + j]
    assert out.shape == ref.shape
    assert np.allclose(out, ref, rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------ tolerance metric
def test_row_rel_err_by_hand():
    # row 0: |got - ref| max = 0.5 (at ref 100), row maximum of |ref| = 100       -> 0.005
    # row 1: |got - ref| max = 0.002 (at ref 0.01), row maximum of |ref| = 0.02   -> 0.1
    # row 2: reference all zero -> denominator 1                                   -> 0.25
    # A per-array maximum would give (0.005, 2e-5, 0.0025); |got| in the denominator (100.5, 0.021, 0.25) would
    # give (0.004975.., 0.0952.., 1.0); a mean instead of a maximum, or an element-wise ratio, differs as well.
    from oracle import row_rel_err
    ref = np.array([[100.0, -1.0, 0.0], [0.01, -0.02, 0.0], [0.0, 0.0, 0.0]])
    got = np.array([[100.5, -1.25, 0.0], [0.012, -0.021, 0.001], [0.0, -0.25, 0.125]])
    err = row_rel_err(got, ref)
    assert err.shape == (3,)
    assert np.allclose(err, [0.005, 0.1, 0.25], rtol=1e-12, atol=0)
    # symmetric in the sign of the error, zero for equal arrays, and rows do not influence one another
    assert np.allclose(row_rel_err(2 * ref - got, ref), err, rtol=1e-9)
    assert np.array_equal(row_rel_err(ref, ref), np.zeros(3))
    assert np.allclose(row_rel_err(got[1:2], ref[1:2]), [0.1], rtol=1e-12)
    assert row_rel_err(np.zeros((0, 3)), np.zeros((0, 3))).shape == (0,)
