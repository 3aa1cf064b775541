"""Pins for the oracle's backward of the centroid and restore steps.  The paper
gives no formula for it, so the reference is the chain rule; it is pinned to
central finite differences of the oracle's own forward functions (evaluated
without rounding), to closed forms and to invariants."""
import numpy as np
import pytest

from oracle import (group_ref, centroid_ref, restore_ref, restore_backward_ref, compress_backward_ref,
                    combine_backward_ref, narrow, widen)


def _setup(seed, T=40, d=6, k=2, E=3, nb=14):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    expert = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    bucket = rng.integers(0, nb, size=T).astype(np.uint64)
    g = group_ref(expert, bucket, E)
    A = rng.standard_normal((E, d, d)) * 0.5          # one small nonlinear "expert" per destination
    b = rng.standard_normal((E, d)) * 0.1
    W = rng.standard_normal((T * k, d))               # loss = sum(W * Y)
    return x, g, A, b, W, k


def _expert(c, g, A, b):
    e = g["seg_expert"].astype(np.int64)
    return np.tanh(np.einsum("sd,sde->se", c, A[e]) + b[e])


def _forward_loss(x, g, A, b, W, k, no_residual):
    c = centroid_ref(x, g["perm"], g["seg_offsets"], k, "f64")
    ec = _expert(c, g, A, b)
    y = restore_ref(x, c, ec, g["seg_of"], k, "f64", no_residual=no_residual)
    return float((W * y).sum())


@pytest.mark.parametrize("no_residual", [False, True])
@pytest.mark.parametrize("seed", [0, 1])
def test_backward_matches_central_differences_of_the_forward(seed, no_residual):
    x, g, A, b, W, k = _setup(seed)
    assert (np.diff(g["seg_offsets"]) > 1).any() and (np.diff(g["seg_offsets"]) == 1).any()
    # analytic chain: dL/dY = W -> dL/dEC (segment sums) -> expert backward -> dL/dx
    G = restore_backward_ref(W, g["perm"], g["seg_offsets"], "f64")
    c = centroid_ref(x, g["perm"], g["seg_offsets"], k, "f64")
    ec = _expert(c, g, A, b)
    e = g["seg_expert"].astype(np.int64)
    h = np.einsum("se,sde->sd", (1.0 - ec ** 2) * G, A[e])
    gx = compress_backward_ref(W, h, G, g["seg_of"], g["seg_offsets"], k, "f64", no_residual=no_residual)
    eps = 1e-6
    num = np.empty_like(x)
    for t in range(x.shape[0]):
        for i in range(x.shape[1]):
            xp, xm = x.copy(), x.copy()
            xp[t, i] += eps
            xm[t, i] -= eps
            num[t, i] = (_forward_loss(xp, g, A, b, W, k, no_residual) - _forward_loss(xm, g, A, b, W, k, no_residual)) / (2 * eps)
    assert np.abs(gx - num).max() < 1e-7 * max(1.0, np.abs(num).max())


def test_segment_sum_against_a_python_loop():
    x, g, A, b, W, k = _setup(2)
    G = restore_backward_ref(W, g["perm"], g["seg_offsets"], "f64")
    for s in range(g["S"]):
        members = [a for a in range(W.shape[0]) if g["seg_of"][a] == s]
        assert np.allclose(G[s], sum(W[a] for a in members), rtol=0, atol=1e-12)


def test_one_member_clusters_pass_the_expert_gradient_through():
    # every assignment alone in its cluster: Y_a = E(x_a), so dL/dx_t = sum_j of the expert's input gradients
    T, d, k, E = 30, 5, 2, 4
    rng = np.random.default_rng(3)
    expert = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    g = group_ref(expert, np.arange(T, dtype=np.uint64), E)
    assert g["S"] == T * k
    gy = rng.standard_normal((T * k, d))
    h = rng.standard_normal((T * k, d))
    G = restore_backward_ref(gy, g["perm"], g["seg_offsets"], "f64")
    assert np.array_equal(G[g["seg_of"]], gy)
    gx = compress_backward_ref(gy, h, G, g["seg_of"], g["seg_offsets"], k, "f64")
    assert np.allclose(gx, h[g["seg_of"]].reshape(T, k, d).sum(axis=1), rtol=0, atol=1e-12)


def test_identity_expert_gives_the_plain_sum_of_output_gradients():
    # E(c) = c makes Y_a = x_a whatever the clustering, so dL/dx_t = sum_j dL/dY_a; the expert backward is h = G
    x, g, A, b, W, k = _setup(4, T=60, nb=3)
    G = restore_backward_ref(W, g["perm"], g["seg_offsets"], "f64")
    gx = compress_backward_ref(W, G, G, g["seg_of"], g["seg_offsets"], k, "f64")
    assert np.allclose(gx, W.reshape(-1, k, W.shape[1]).sum(axis=1), rtol=0, atol=1e-12)


def test_gradient_mass_is_conserved():
    # sum_t dL/dx_t = sum_s h_s: the residual terms cancel inside every cluster
    x, g, A, b, W, k = _setup(5, T=80, nb=7)
    h = np.random.default_rng(6).standard_normal((g["S"], x.shape[1]))
    G = restore_backward_ref(W, g["perm"], g["seg_offsets"], "f64")
    for flag in (False, True):
        gx = compress_backward_ref(W, h, G, g["seg_of"], g["seg_offsets"], k, "f64", no_residual=flag)
        assert np.allclose(gx.sum(axis=0), h.sum(axis=0), rtol=0, atol=1e-10)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_storage_types_round_once(dtype):
    x, g, A, b, W, k = _setup(7)
    Ws = narrow(W, dtype)
    G = restore_backward_ref(Ws, g["perm"], g["seg_offsets"], dtype)
    G64 = restore_backward_ref(widen(Ws, dtype), g["perm"], g["seg_offsets"], "f64")
    assert np.array_equal(G, narrow(G64, dtype))
    h = narrow(np.random.default_rng(8).standard_normal(G64.shape), dtype)
    gx = compress_backward_ref(Ws, h, G, g["seg_of"], g["seg_offsets"], k, dtype)
    gx64 = compress_backward_ref(widen(Ws, dtype), widen(h, dtype), widen(G, dtype), g["seg_of"], g["seg_offsets"], k, "f64")
    assert np.array_equal(gx, narrow(gx64, dtype))


# ------------------------------------------------------------------ backward of the gate-weighted combine
def test_combine_backward_by_hand():
    # the hand-worked forward case of the restore pins: two tokens, experts (0, 1) each, one bucket:
    #   Y[a0] = (9, 22), Y[a1] = (99, 202), Y[a2] = (11, 18), Y[a3] = (101, 198); w = [[0.25, 0.5], [2, -1]]
    # with dL/dout = [[1, 2], [3, -1]]:
    #   dL/dw = [[1*9 + 2*22, 1*99 + 2*202], [3*11 - 18, 3*101 - 198]] = [[53, 503], [15, 105]]
    #   dL/dY = [0.25*(1, 2), 0.5*(1, 2), 2*(3, -1), -1*(3, -1)]
    x = np.array([[1.0, 7.0], [3.0, 3.0]], np.float32)
    expert = np.array([[0, 1], [0, 1]], np.int32)
    g = group_ref(expert, np.zeros(2, np.uint64), 2)
    c = centroid_ref(x, g["perm"], g["seg_offsets"], 2, "f32")
    ec = np.array([[10.0, 20.0], [100.0, 200.0]], np.float32)
    w = np.array([[0.25, 0.5], [2.0, -1.0]], np.float32)
    go = np.array([[1.0, 2.0], [3.0, -1.0]], np.float32)
    gw, gy = combine_backward_ref(x, c, ec, g["seg_of"], 2, "f32", w, go)
    assert gw.tolist() == [[53.0, 503.0], [15.0, 105.0]]
    assert gy.tolist() == [[0.25, 0.5], [0.5, 1.0], [6.0, -2.0], [-3.0, 1.0]]
    # without the residual Y[a] = EC[s]: dL/dw = [[10 + 40, 100 + 400], [30 - 20, 300 - 200]]
    gw0, gy0 = combine_backward_ref(x, c, ec, g["seg_of"], 2, "f32", w, go, no_residual=True)
    assert gw0.tolist() == [[50.0, 500.0], [10.0, 100.0]]
    assert np.array_equal(gy0, gy)


def _combined_loss(x, w, g, A, b, Wt, k, no_residual):
    c = centroid_ref(x, g["perm"], g["seg_offsets"], k, "f64")
    ec = _expert(c, g, A, b)
    out = restore_ref(x, c, ec, g["seg_of"], k, "f64", no_residual=no_residual, gate_weight=w)   # [T, d]
    return float((Wt * out).sum())


@pytest.mark.parametrize("no_residual", [False, True])
def test_combine_backward_matches_central_differences(no_residual):
    # loss = sum(Wt * out), out = gate-weighted combine of the restored rows; gradients for the gate weights and,
    # through restore_backward_ref / the expert / compress_backward_ref, for the tokens
    x, g, A, b, W, k = _setup(11)
    T, d = x.shape
    rng = np.random.default_rng(12)
    w = rng.standard_normal((T, k))
    Wt = rng.standard_normal((T, d))
    c = centroid_ref(x, g["perm"], g["seg_offsets"], k, "f64")
    ec = _expert(c, g, A, b)
    gw, gy = combine_backward_ref(x, c, ec, g["seg_of"], k, "f64", w, Wt, no_residual=no_residual)
    G = restore_backward_ref(gy, g["perm"], g["seg_offsets"], "f64")
    e = g["seg_expert"].astype(np.int64)
    h = np.einsum("se,sde->sd", (1.0 - ec ** 2) * G, A[e])
    gx = compress_backward_ref(gy, h, G, g["seg_of"], g["seg_offsets"], k, "f64", no_residual=no_residual)
    eps = 1e-6
    num_w = np.empty_like(w)
    for t in range(T):
        for j in range(k):
            wp, wm = w.copy(), w.copy()
            wp[t, j] += eps
            wm[t, j] -= eps
            num_w[t, j] = (_combined_loss(x, wp, g, A, b, Wt, k, no_residual) - _combined_loss(x, wm, g, A, b, Wt, k, no_residual)) / (2 * eps)
    assert np.abs(gw - num_w).max() < 1e-7 * max(1.0, np.abs(num_w).max())
    num_x = np.empty_like(x)
    for t in range(T):
        for i in range(d):
            xp, xm = x.copy(), x.copy()
            xp[t, i] += eps
            xm[t, i] -= eps
            num_x[t, i] = (_combined_loss(xp, w, g, A, b, Wt, k, no_residual) - _combined_loss(xm, w, g, A, b, Wt, k, no_residual)) / (2 * eps)
    assert np.abs(gx - num_x).max() < 1e-7 * max(1.0, np.abs(num_x).max())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_combine_backward_rounds_the_row_gradient_once_and_leaves_the_weight_gradient_unrounded(dtype):
    x, g, A, b, W, k = _setup(13)
    T, d = x.shape
    rng = np.random.default_rng(14)
    xs = narrow(x, dtype)
    c = centroid_ref(xs, g["perm"], g["seg_offsets"], k, dtype)
    ec = narrow(rng.standard_normal((g["S"], d)), dtype)
    w = rng.standard_normal((T, k)).astype(np.float32)
    go = narrow(rng.standard_normal((T, d)), dtype)
    gw, gy = combine_backward_ref(xs, c, ec, g["seg_of"], k, dtype, w, go)
    gw64, gy64 = combine_backward_ref(widen(xs, dtype), widen(c, dtype), widen(ec, dtype), g["seg_of"], k, "f64",
                                      w.astype(np.float64), widen(go, dtype))
    assert gw.dtype == np.float64 and np.array_equal(gw, gw64)
    assert np.array_equal(gy, narrow(gy64, dtype))
    # weights of one: the row gradient is the output gradient repeated k times
    _, gy1 = combine_backward_ref(xs, c, ec, g["seg_of"], k, dtype, np.ones((T, k), np.float32), go)
    assert np.array_equal(gy1, np.repeat(go, k, axis=0))
