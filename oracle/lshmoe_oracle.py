"""CPU oracle for the LSH-MoE token compression / restoration path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP kernels are checked against.  It may be imported by tests, by the smoke
check and by the benchmark's cpu-baseline leg, and by nothing else; it shares
no code, table or helper with the HIP path and never imports it.

Everything is computed in IEEE binary64 on the exactly-widened inputs and
rounded once to the storage type at the end of each step.  Library primitives
used as steps: numpy matmul (the rotation), numpy lexsort (the stable sort),
numpy add.reduceat (the per-bucket sums).

Storage convention for arrays: "f32" = numpy float32, "bf16" = numpy uint16
holding the upper half of the binary32 pattern, "f64" = numpy float64 (no
rounding at all; used by the finite-difference pins of the backward pass).

Pins (tests/test_oracle_*.py): pure-Python brute force on tiny inputs, the
cross-polytope invariants (positive scaling, negation, row permutation of R),
identity / orthonormal closed forms, dict- and numpy.unique-based grouping,
mass conservation, exact reconstruction for singleton buckets, the linear
expert closed form, hand-worked gate-weighted combines (shared two-member
clusters, unequal weights) and the weighted-sum identity over the unweighted
rows, a hand-worked case of the row-scaled error metric; for the backward pass
central finite differences of the forward functions of this file (also through
the gate-weighted combine, for tokens and for gate weights), its closed forms
for one-member clusters and for an identity expert, a hand-worked combine
gradient, and gradient mass conservation.  Absolute values of
the whole path on the synthetic workloads have no printed counterpart in the
paper: beyond those pins they are parity unpinned.  sphere_hash_ref follows a
reading of a hash family that the paper only names (Section 4.5): it is pinned
to its own definition (exact integer brute force, translation invariance,
radius monotonicity, the hyperplane limit, bit order by hand) and stays
parity unpinned against the paper.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# storage <-> binary64
# --------------------------------------------------------------------------
def widen(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact conversion of a storage array to float64."""
    if dtype == "f64":
        assert x.dtype == np.float64
        return x
    if dtype == "f32":
        assert x.dtype == np.float32
        return x.astype(np.float64)
    if dtype == "bf16":
        assert x.dtype == np.uint16
        bits = x.astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def narrow(x64: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 to the storage type: binary64 -> binary32 with
    round-to-nearest-even, then (bf16 only) binary32 -> bfloat16 with
    round-to-nearest-even on the discarded 16 bits.  Finite inputs only.
    "f64" keeps the values as they are."""
    if dtype == "f64":
        return np.asarray(x64, dtype=np.float64)
    f32 = np.asarray(x64, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return f32
    if dtype == "bf16":
        u = np.ascontiguousarray(f32).view(np.uint32).astype(np.uint64)
        kept_lsb = (u >> np.uint64(16)) & np.uint64(1)
        u = u + np.uint64(0x7FFF) + kept_lsb
        return (u >> np.uint64(16)).astype(np.uint16)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# Step 1 - cross-polytope hash (Section 3.2, Eq. 3; Alg. 1 "LSH(X_i)")
# --------------------------------------------------------------------------
def hash_ref(tokens: np.ndarray, rot: np.ndarray, dtype: str):
    """Cross-polytope bucket of every token.

    tokens [T, d], rot [L, r, d] in storage form.  For hash l the rotated
    vector is y = R_l x (r coordinates).  The nearest of the 2r cross-polytope
    vertices +-e_i is the coordinate of largest |y_i| together with the sign
    of y there: code = i* if y[i*] >= 0 else i* + r, with the lowest index
    winning among equal magnitudes.  The L codes are combined as the digits of
    a base-2r number, hash 0 most significant.

    Returns (bucket uint64 [T], code int32 [T, L], margin float64 [T, L],
    runner_up int32 [T, L]).  margin = (m1 - m2) / m1 for the two largest
    magnitudes m1 >= m2 (0 when m1 == 0); runner_up is the code the second
    largest coordinate would give.  The last two exist so that a comparison
    with a lower-precision implementation can recognise near ties.
    """
    L, r, d = rot.shape
    T = tokens.shape[0]
    assert tokens.shape == (T, d)
    assert r >= 2 and (2 * r) ** L < 2 ** 63
    x = widen(tokens, dtype)                       # [T, d]
    R = widen(rot, dtype)                          # [L, r, d]
    code = np.empty((T, L), np.int32)
    margin = np.empty((T, L), np.float64)
    runner = np.empty((T, L), np.int32)
    rows = np.arange(T)
    for l in range(L):
        y = x @ R[l].T                             # [T, r]  y[t, i] = <R_l[i, :], x_t>
        mag = np.abs(y)
        i1 = np.argmax(mag, axis=1)                # first index attaining the maximum
        m1 = mag[rows, i1]
        code[:, l] = i1 + np.where(y[rows, i1] < 0.0, r, 0)
        mag2 = mag.copy()
        mag2[rows, i1] = -1.0
        i2 = np.argmax(mag2, axis=1)
        m2 = mag[rows, i2]
        runner[:, l] = i2 + np.where(y[rows, i2] < 0.0, r, 0)
        with np.errstate(invalid="ignore", divide="ignore"):
            margin[:, l] = np.where(m1 > 0.0, (m1 - m2) / np.where(m1 > 0.0, m1, 1.0), 0.0)
    bucket = combine_codes(code, r)
    return bucket, code, margin, runner


def gate_logits_ref(tokens: np.ndarray, gate_w: np.ndarray, dtype: str) -> np.ndarray:
    """Linear part of a learned gate (the gating network of Section 2.1, Eq. 1,
    whose form the paper leaves open): logits[t, e] = <gate_w[e, :], x_t>,
    in binary64, not rounded.  tokens [T, d], gate_w [E, d] in storage form."""
    return widen(tokens, dtype) @ widen(gate_w, dtype).T


def sphere_hash_ref(tokens: np.ndarray, pivots: np.ndarray, radius_sq: np.ndarray, dtype: str):
    """Spherical hashing, the alternative hash family of the ablation in Section 4.5 ("SP").  The paper names
    it without defining it; the reading taken here is the hypersphere-based binary code of spherical hashing:
    hash function l is a sphere with centre pivots[l] and squared radius radius_sq[l], and
        bit_l(x) = 1  if  ||x - p_l||^2 <= radius_sq[l]  (inside or on the sphere),  else 0.
    The B bits form the bucket id, bit 0 most significant (as the digits of the cross-polytope hash).  Far pivots
    with large radii make the spheres locally flat, which is how the family contains hyperplane hashing.

    tokens [T, d], pivots [B, d] in storage form, radius_sq [B] float (any real values, B <= 63).
    Returns (bucket uint64 [T], bit uint8 [T, B], margin float64 [T, B]) with
    margin = | ||x - p_l||^2 - radius_sq[l] | / max(|radius_sq[l]|, ||x - p_l||^2): how far, relatively, the token is
    from the decision surface, so that a lower-precision implementation can recognise borderline bits."""
    B, d = pivots.shape
    T = tokens.shape[0]
    assert tokens.shape == (T, d) and radius_sq.shape == (B,) and 1 <= B <= 63
    x = widen(tokens, dtype)
    p = widen(pivots, dtype)
    t2 = np.asarray(radius_sq, dtype=np.float64)
    bit = np.empty((T, B), np.uint8)
    margin = np.empty((T, B), np.float64)
    for l in range(B):
        diff = x - p[l]                              # [T, d]
        dist2 = (diff * diff).sum(axis=1)
        bit[:, l] = dist2 <= t2[l]
        scale = np.maximum(np.abs(t2[l]), dist2)
        margin[:, l] = np.abs(dist2 - t2[l]) / np.where(scale > 0.0, scale, 1.0)
    bucket = np.zeros(T, np.uint64)
    for l in range(B):
        bucket = bucket * np.uint64(2) + bit[:, l].astype(np.uint64)
    return bucket, bit, margin


def combine_codes(code: np.ndarray, r: int) -> np.ndarray:
    """Digits code[:, 0..L-1] (each in [0, 2r)) -> one base-2r number, digit 0
    most significant."""
    T, L = code.shape
    bucket = np.zeros(T, np.uint64)
    for l in range(L):
        bucket = bucket * np.uint64(2 * r) + code[:, l].astype(np.uint64)
    return bucket


# --------------------------------------------------------------------------
# Step 2 - group assignments by (expert, bucket)  (Alg. 1: dispatch, then
# "divide X_i into clusters based on IDX")
# --------------------------------------------------------------------------
def group_ref(expert: np.ndarray, bucket: np.ndarray, E: int):
    """Assignment a = t*k + j (token t, its j-th expert) has key
    (expert[t, j], bucket[t]).  Clusters are the sets of assignments with
    equal key; they are listed by ascending (expert, bucket) and, inside a
    cluster, by ascending a.

    Returns a dict:
      perm           int32 [N]    sorted position -> assignment
      seg_offsets    int32 [S+1]  cluster s covers perm[seg_offsets[s]:seg_offsets[s+1]]
      seg_expert     int32 [S]    destination expert of cluster s
      expert_offsets int32 [E+1]  clusters of expert e are [expert_offsets[e], expert_offsets[e+1])
      seg_of         int32 [N]    assignment -> cluster
      S              int
    """
    T, k = expert.shape
    N = T * k
    ea = expert.reshape(N).astype(np.int64)
    ba = np.repeat(bucket.astype(np.uint64), k)
    perm = np.lexsort((ba, ea))                    # stable; last key is primary
    es, bs = ea[perm], ba[perm]
    head = np.ones(N, bool)
    head[1:] = (es[1:] != es[:-1]) | (bs[1:] != bs[:-1])
    starts = np.flatnonzero(head)
    S = int(starts.size)
    seg_offsets = np.concatenate([starts, [N]]).astype(np.int32)
    seg_expert = es[starts].astype(np.int32)
    seg_id_sorted = np.cumsum(head) - 1
    seg_of = np.empty(N, np.int32)
    seg_of[perm] = seg_id_sorted
    expert_offsets = np.searchsorted(seg_expert, np.arange(E + 1), side="left").astype(np.int32)
    return dict(perm=perm.astype(np.int32), seg_offsets=seg_offsets, seg_expert=seg_expert,
                expert_offsets=expert_offsets, seg_of=seg_of, S=S)


# --------------------------------------------------------------------------
# Step 3 - centroids  (Section 2.3 centroid formula with 1/n_j; Alg. 1 "Mean")
# --------------------------------------------------------------------------
def centroid_ref(tokens: np.ndarray, perm: np.ndarray, seg_offsets: np.ndarray, k: int, dtype: str,
                 return_f64: bool = False):
    """c_s = (1/n_s) * sum of the token rows of cluster s, rounded once to
    the storage type.  Row of assignment a is tokens[a // k]."""
    S = seg_offsets.size - 1
    x = widen(tokens, dtype)
    rows = x[perm.astype(np.int64) // k]           # [N, d] in sorted order
    sums = np.add.reduceat(rows, seg_offsets[:-1].astype(np.int64), axis=0) if S > 0 \
        else np.zeros((0, x.shape[1]))
    n = np.diff(seg_offsets.astype(np.int64)).astype(np.float64)
    c64 = sums / n[:, None]
    if return_f64:
        return narrow(c64, dtype), c64
    return narrow(c64, dtype)


# --------------------------------------------------------------------------
# Step 4 - restore with residual compensation  (Eq. 4 and Eq. 5; Alg. 1 last loop)
# --------------------------------------------------------------------------
def restore_ref(tokens: np.ndarray, centroids: np.ndarray, expert_out: np.ndarray, seg_of: np.ndarray,
                k: int, dtype: str, no_residual: bool = False, gate_weight: np.ndarray | None = None):
    """Y[a] = E(c_s) + (x_a - c_s) with s = seg_of[a]; the residual is taken
    against the stored (rounded) centroid, so a one-member cluster returns
    E(c_s) exactly.  no_residual drops the compensation term (the ablation
    arm of Fig. 5).  With gate_weight [T, k] the k rows of a token are
    combined as sum_j w[t, j] * Y[t*k + j] (Eq. 2 with gate weights) and the
    result is [T, d]; otherwise it is [N, d]."""
    s = seg_of.astype(np.int64)
    N = s.size
    ec = widen(expert_out, dtype)[s]
    if no_residual:
        y = ec
    else:
        x = widen(tokens, dtype)[np.arange(N) // k]
        c = widen(centroids, dtype)[s]
        y = ec + (x - c)
    if gate_weight is not None:
        T = N // k
        w = gate_weight.astype(np.float64).reshape(T, k, 1)
        y = (w * y.reshape(T, k, -1)).sum(axis=1)
    return narrow(y, dtype)


# --------------------------------------------------------------------------
# Backward of steps 3 and 4.  The paper does not describe it (it counts the
# backward all-to-alls in Section 3.1 but says nothing of how gradients pass
# through the compression); this is the chain rule applied to
#     c_s = (1/n_s) sum_{a in s} x_a,   Y_a = EC_s + (x_a - c_s)
# with the cluster membership held fixed.
# --------------------------------------------------------------------------
def restore_backward_ref(grad_out: np.ndarray, perm: np.ndarray, seg_offsets: np.ndarray, dtype: str):
    """Gradient with respect to the expert outputs: EC_s reaches every member
    row unchanged, so dL/dEC_s = sum_{a in s} grad_out[a].  grad_out is
    [N, d] in assignment order; the result is [S, d], rounded once."""
    S = seg_offsets.size - 1
    g = widen(grad_out, dtype)
    rows = g[perm.astype(np.int64)]                # [N, d] in sorted order
    sums = np.add.reduceat(rows, seg_offsets[:-1].astype(np.int64), axis=0) if S > 0 \
        else np.zeros((0, g.shape[1]))
    return narrow(sums, dtype)


def compress_backward_ref(grad_out: np.ndarray, grad_centroids: np.ndarray, grad_expert_out: np.ndarray,
                          seg_of: np.ndarray, seg_offsets: np.ndarray, k: int, dtype: str,
                          no_residual: bool = False):
    """Gradient with respect to the tokens.  grad_centroids[s] is what the
    expert's backward returns for its input c_s; grad_expert_out[s] is the
    stored result of restore_backward_ref.  The centroid enters Y_a of every
    member with coefficient -1, so the total gradient of c_s is
    grad_centroids[s] - grad_expert_out[s], and c_s depends on each member
    with weight 1/n_s:
        dL/dx_t = sum_j ( grad_out[a] + (grad_centroids[s] - grad_expert_out[s]) / n_s ),
        a = t*k + j, s = seg_of[a].
    Without the residual term (no_residual) Y_a = EC_s and only
    grad_centroids[s] / n_s remains.  Result [T, d], rounded once."""
    s = seg_of.astype(np.int64)
    N = s.size
    T = N // k
    n = np.diff(seg_offsets.astype(np.int64)).astype(np.float64)[s][:, None]
    h = widen(grad_centroids, dtype)[s]
    if no_residual:
        per_a = h / n
    else:
        per_a = widen(grad_out, dtype) + (h - widen(grad_expert_out, dtype)[s]) / n
    return narrow(per_a.reshape(T, k, -1).sum(axis=1), dtype)


def combine_backward_ref(tokens: np.ndarray, centroids: np.ndarray, expert_out: np.ndarray, seg_of: np.ndarray,
                         k: int, dtype: str, gate_weight: np.ndarray, grad_out: np.ndarray,
                         no_residual: bool = False):
    """Backward of the gate-weighted combine of restore_ref(gate_weight=...) (Eq. 2 with gate weights over
    Eq. 4 / Eq. 5):  out[t] = sum_j w[t, j] * Y[t*k + j]  is linear in the weights and in the restored rows, so
        dL/dw[t, j]   = < grad_out[t, :], Y[t*k + j, :] >          (the gate's gradient; float64, not rounded)
        dL/dY[t*k+j]  = w[t, j] * grad_out[t, :]                    (rounded once to the storage type)
    with Y[a] = E(c_s) + (x_a - c_s) (or E(c_s) without the residual) evaluated, as in the forward, from the stored
    centroids and never rounded itself.  dL/dY is what restore_backward_ref and compress_backward_ref take as
    their grad_out.  grad_out is [T, d] in storage form, gate_weight [T, k]."""
    s = seg_of.astype(np.int64)
    N = s.size
    T = N // k
    y = widen(expert_out, dtype)[s]
    if not no_residual:
        y = y + (widen(tokens, dtype)[np.arange(N) // k] - widen(centroids, dtype)[s])
    g = widen(grad_out, dtype)                        # [T, d]
    grad_w = np.einsum("td,tkd->tk", g, y.reshape(T, k, -1))
    w = gate_weight.astype(np.float64).reshape(T, k, 1)
    grad_y = (w * g[:, None, :]).reshape(N, -1)
    return grad_w, narrow(grad_y, dtype)


# --------------------------------------------------------------------------
# whole path, for timing and smoke checks
# --------------------------------------------------------------------------
def row_rel_err(got64: np.ndarray, ref64: np.ndarray) -> np.ndarray:
    """Per-row error max_j |got - ref| / max_j |ref| (rows whose reference is
    all zero use denominator 1)."""
    num = np.abs(got64 - ref64).max(axis=1) if got64.shape[1] else np.zeros(got64.shape[0])
    den = np.abs(ref64).max(axis=1) if ref64.shape[1] else np.ones(ref64.shape[0])
    return num / np.where(den > 0.0, den, 1.0)
