/*
 * lshmoe.h - C ABI of the MI355X (gfx950) LSH-MoE token compression library.
 *
 * The library implements the per-GPU work that LSH-MoE places around the MoE
 * all-to-all (Section 3.2; Algorithm 1 in the appendix):
 *
 *   lshmoe_hash        cross-polytope LSH of every token            (Eq. 3)
 *   lshmoe_compress    cluster each expert's tokens by bucket and
 *                      replace every cluster by its centroid        (Alg. 1, the two nested loops)
 *   lshmoe_decompress  give every token the expert output of its
 *                      centroid plus the token's residual           (Eq. 4, Eq. 5)
 *   lshmoe_hash_sphere          the spherical hash family of the ablation (Section 4.5), one bit per sphere
 *   lshmoe_hash_gate            lshmoe_hash that also returns the gate's projection of the tokens (Eq. 1)
 *   lshmoe_decompress_combine   lshmoe_decompress fused with the gate-weighted sum over a token's experts (Eq. 2)
 *   lshmoe_decompress_backward, lshmoe_compress_backward   gradients through the two calls above
 *   lshmoe_decompress_combine_backward                      gradients of the fused combine (gate weights and rows)
 *   lshmoe_compress_static      lshmoe_compress on scratch memory built into the library (allocates nothing)
 *
 * Notation: T tokens of dimension d; every token is routed to k distinct
 * experts out of E (assignment a = t*k + j is token t's j-th expert, N = T*k
 * assignments); L hash functions, each a real matrix R_l with r rows (so 2r
 * buckets per hash and (2r)^L combined buckets); S clusters ("segments"), one
 * per non-empty (expert, bucket) pair.
 *
 * Conventions for every entry point
 *   - All array pointers are DEVICE pointers owned by the caller, row-major,
 *     contiguous, 16-byte aligned.  Inputs are never written; outputs must not
 *     overlap inputs or each other.  The library keeps no pointer after a call
 *     returns and allocates no device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it and return; nothing synchronises the host.
 *     That is why the cluster count S stays in device memory and outputs are
 *     sized for the worst case S == N.
 *   - dtype LSHMOE_F32 is IEEE binary32; LSHMOE_BF16 is bfloat16 (upper 16 bits
 *     of binary32).  All sums are accumulated in binary32 and rounded to the
 *     storage type once, round-to-nearest-even.
 *   - The row size d * sizeof(element) must be a multiple of 16 bytes.
 *   - Entry points that move [N, d] rows (compress, decompress, the backward
 *     pair) address 16-byte pieces with 32-bit indices inside one launch:
 *     N * d * sizeof(element) / 16 must not exceed 2^32 - 256, i.e. about 64 GiB
 *     of rows per call (LSHMOE_ERR_UNSUPPORTED beyond).
 *   - Return value: LSHMOE_OK or an error code; nothing is enqueued on a host
 *     side error.  lshmoe_last_error() gives a thread-local description.
 *     Arguments are checked on the host before any GPU call, so the checks
 *     behave the same on a machine without a GPU.
 *   - Preconditions that are NOT checked (results are unspecified, memory
 *     safety is kept for out-of-range expert ids, which count as E - 1, and
 *     for bucket ids wider than (2r)^L - 1, whose extra bits are dropped): finite
 *     inputs; 0 <= expert[t][j] < E; the k experts of one token are distinct;
 *     bucket ids as lshmoe_hash writes them for the same L and r.
 */
#ifndef LSHMOE_H
#define LSHMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LSHMOE_OK = 0,
  LSHMOE_ERR_NULL = 1,        /* a required pointer is NULL                         */
  LSHMOE_ERR_SHAPE = 2,       /* a size is non-positive or inconsistent (k > E ...) */
  LSHMOE_ERR_UNSUPPORTED = 3, /* valid but outside what the kernels handle          */
  LSHMOE_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small         */
  LSHMOE_ERR_HIP = 5          /* a HIP runtime call failed                          */
} lshmoe_status;

typedef enum {
  LSHMOE_F32 = 0,
  LSHMOE_BF16 = 1,
  LSHMOE_DTYPE_INT_RANGE_ = 0x7fffffff /* not a dtype: makes every int a representable value, so that an unknown
                                          code from a caller is an error return (LSHMOE_ERR_UNSUPPORTED), never
                                          undefined behaviour inside the library */
} lshmoe_dtype;

/* Flags of lshmoe_decompress. */
enum {
  /* Drop the residual term: Y = E(centroid).  The paper's "without error
   * compensation" arm (Section 4.2, Fig. 5). */
  LSHMOE_FLAG_NO_RESIDUAL = 1u
};

/* Static, never-freed name of a status code. */
const char* lshmoe_status_string(int status);

/* Description of the last error raised on the calling thread ("" if none).
 * Valid until the next library call on that thread. */
const char* lshmoe_last_error(void);

/* ABI version of this header (bumped when a signature changes). */
int lshmoe_abi_version(void);

/*
 * Bytes of device scratch lshmoe_compress needs for these sizes (host only,
 * touches no GPU).  Errors: NULL out_bytes; non-positive sizes; k > E;
 * unsupported sizes as for lshmoe_compress.
 */
lshmoe_status lshmoe_workspace_bytes(int64_t T, int32_t d, int32_t k, int32_t E,
                                     int32_t L, int32_t r, lshmoe_dtype dtype,
                                     size_t* out_bytes);

/*
 * Cross-polytope hash (Section 3.2, Eq. 3).  For hash l the token x is mapped
 * to y = R_l x (r coordinates) and then to the nearest vertex of the
 * cross-polytope {+-e_i}: code_l = i* if y[i*] >= 0 else i* + r, where i* is
 * the lowest index attaining max_i |y_i|.  The L codes are the digits of a
 * base-2r number, hash 0 most significant:
 *     bucket[t] = ((code_0 * 2r + code_1) * 2r + ...) * 2r + code_{L-1}.
 * R_l may be any real r x d matrix (a rotation restricted to r rows is the
 * intended use; orthonormality is not required or checked).
 *
 *   tokens [T, d]   in   dtype
 *   rot    [L, r, d] in  dtype
 *   bucket [T]      out  uint64
 *
 * The products are exact in binary32 for bf16 inputs and are accumulated in
 * binary32 (16 products per matrix instruction), so every y_i carries an error
 * of at most (d/16 + 8) * 2^-24 * sum_j |R_l[i][j] x_j|: about 3e-5 of the
 * largest |y_i| for Gaussian data at d = 1024, typically a tenth of that.  A
 * token whose two largest |y_i| differ by less than 1e-4 relative may therefore
 * land on the other of the two vertices than exact arithmetic gives; apart from
 * such near ties the codes are those of exact arithmetic.
 * Errors: NULL pointer; T, d, L, r <= 0; r < 2 or (2r)^L >= 2^63
 * (UNSUPPORTED); r > 256 (UNSUPPORTED); d*sizeof(element) not a multiple of 16
 * (UNSUPPORTED); launch failure (HIP).
 */
lshmoe_status lshmoe_hash(const void* tokens, const void* rot,
                          int64_t T, int32_t d, int32_t L, int32_t r, lshmoe_dtype dtype,
                          uint64_t* bucket, void* stream);

/*
 * Spherical hash: the alternative hash family of the ablation in Section 4.5 ("SP"; Section 3.2 lists it among the
 * LSH algorithms that were tried).  The paper names the family without defining it; this entry point takes it as the
 * hypersphere-based binary code of spherical hashing: sphere l has the centre pivots[l, :] and the squared radius
 * radius_sq[l], and
 *     bit_l(x) = 1  if  |x - p_l|^2 <= radius_sq[l]  (inside or on the sphere),  else 0;
 *     bucket[t] = sum_l bit_l(x_t) * 2^(B-1-l)        (bit 0 most significant).
 * Pivots far away with large radii give locally flat spheres, i.e. hyperplane hashing.  How the spheres are chosen
 * is the caller's business.  The bucket ids feed lshmoe_compress like those of lshmoe_hash; its L and r only have to
 * bound them, (2r)^L >= 2^B: for example r = 2 and L = ceil(B / 2).
 *
 *   tokens    [T, d]  in   dtype
 *   pivots    [B, d]  in   dtype
 *   radius_sq [B]     in   binary32 (any real values; a negative one leaves its sphere empty)
 *   bucket    [T]     out  uint64
 *
 * |x - p|^2 is evaluated as |x|^2 - 2 <p, x> + |p|^2 in binary32 (the dot product on the matrix cores), so a token
 * whose squared distance is within about 1e-4 relative of the squared radius may get the other bit than exact
 * arithmetic gives.
 * Errors: NULL pointer; T, d, B <= 0; B > 63 (UNSUPPORTED); d*sizeof(element) not a multiple of 16 (UNSUPPORTED);
 * T >= 2^30 (UNSUPPORTED); launch failure (HIP).
 */
lshmoe_status lshmoe_hash_sphere(const void* tokens, const void* pivots, const float* radius_sq,
                                 int64_t T, int32_t d, int32_t B, lshmoe_dtype dtype,
                                 uint64_t* bucket, void* stream);

/*
 * lshmoe_hash fused with the linear part of a learned gate (the gating network G of Section 2.1, Eq. 1; the
 * paper leaves its form open; routers "via learnable weighting" start from a projection of the token):
 *     logits[t, e] = < gate_w[e, :], tokens[t, :] >,   accumulated in binary32,
 * computed by the same kernel and from the same read of the tokens as the bucket ids whenever
 * L*r + E <= 128, or L*r <= 256 and E <= 64 on at least 32768 tokens (otherwise the tokens are read a second time
 * for the gate rows).  Choosing the top-k experts from the logits stays with the caller.
 *
 *   gate_w [E, d]  in   dtype
 *   logits [T, E]  out  binary32
 *   other arguments and the bucket ids exactly as for lshmoe_hash.
 *
 * Errors: as for lshmoe_hash; NULL gate_w or logits; E <= 0 (SHAPE); shapes the fused kernel does not take
 * (UNSUPPORTED): r not a multiple of 8, d*sizeof(element) not a multiple of 512, E > 128.
 */
lshmoe_status lshmoe_hash_gate(const void* tokens, const void* rot, const void* gate_w,
                               int64_t T, int32_t d, int32_t L, int32_t r, int32_t E, lshmoe_dtype dtype,
                               uint64_t* bucket, float* logits, void* stream);

/*
 * Cluster and average (Algorithm 1: dispatch by expert, split each expert's
 * tokens into clusters by bucket, take each cluster's mean; centroid formula
 * of Section 2.3 with 1/n_j).
 *
 * Assignment a = t*k + j has key (expert[t][j], bucket[t]).  Clusters are the
 * sets of assignments with equal key, numbered 0..S-1 by ascending
 * (expert, bucket); inside a cluster members are ordered by ascending a.
 *
 *   tokens         [T, d]  in   dtype
 *   expert         [T, k]  in   int32
 *   bucket         [T]     in   uint64, every value < (2r)^L
 *   centroids      [N, d]  out  dtype; rows 0..S-1 are written: the a2a payload
 *   seg_offsets    [N+1]   out  int32; entries 0..S: cluster s owns perm[seg_offsets[s] .. seg_offsets[s+1])
 *   seg_expert     [N]     out  int32; entries 0..S-1: destination expert of cluster s
 *   expert_offsets [E+1]   out  int32; clusters of expert e are [expert_offsets[e], expert_offsets[e+1]):
 *                               the per-destination send counts of the all-to-all
 *   perm           [N]     out  int32; sorted position -> assignment
 *   seg_of         [N]     out  int32; assignment -> cluster
 *   num_segments   [1]     out  int32 (device); S
 *   workspace              scratch of at least lshmoe_workspace_bytes(...) bytes, 256-byte aligned;
 *                          contents on entry are ignored and on return are unspecified
 *
 * L and r only bound the bucket ids (they fix how many key bits are sorted).
 * All integer outputs are deterministic; centroid sums run in member order, so
 * the floating-point result is reproducible bit for bit.
 * Errors: NULL pointer; T, d, k, E, L, r <= 0; k > E; N = T*k >= 2^30
 * (UNSUPPORTED); (2r)^L >= 2^63 or bits(E-1) + bits((2r)^L - 1) > 64
 * (UNSUPPORTED); row size not a multiple of 16 bytes (UNSUPPORTED); workspace
 * too small or misaligned (WORKSPACE); launch failure (HIP).
 */
lshmoe_status lshmoe_compress(const void* tokens, const int32_t* expert, const uint64_t* bucket,
                              int64_t T, int32_t d, int32_t k, int32_t E,
                              int32_t L, int32_t r, lshmoe_dtype dtype,
                              void* centroids, int32_t* seg_offsets, int32_t* seg_expert,
                              int32_t* expert_offsets, int32_t* perm, int32_t* seg_of,
                              int32_t* num_segments,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * lshmoe_compress for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace pair), same
 * kernels and bit-identical outputs; the scratch is an array of LSHMOE_STATIC_SCRATCH_BYTES bytes that is part of
 * the library's device image (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing; its first call on a device looks up that device's address of the array.
 *
 * Sizes whose lshmoe_workspace_bytes exceeds LSHMOE_STATIC_SCRATCH_BYTES are refused with LSHMOE_ERR_WORKSPACE and
 * nothing is enqueued (the five paper-shaped layers of up to T = 65536, d = 1024, k = 2 fit).  All calls on one GPU
 * share the one array: two calls that overlap on that GPU (different streams, or a graph replay beside an eager
 * call) race; calls on one stream are ordered and safe.  What the array holds between calls is unspecified; the
 * kernels clear what they need.
 * Other errors: as for lshmoe_compress; failure to find the array's address (HIP).
 */
#define LSHMOE_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
lshmoe_status lshmoe_compress_static(const void* tokens, const int32_t* expert, const uint64_t* bucket,
                                     int64_t T, int32_t d, int32_t k, int32_t E,
                                     int32_t L, int32_t r, lshmoe_dtype dtype,
                                     void* centroids, int32_t* seg_offsets, int32_t* seg_expert,
                                     int32_t* expert_offsets, int32_t* perm, int32_t* seg_of,
                                     int32_t* num_segments, void* stream);

/*
 * Restore with residual compensation (Eq. 4 and Eq. 5; last loop of
 * Algorithm 1).  For every assignment a with s = seg_of[a]:
 *     out[a, :] = expert_out[s, :] + (tokens[a / k, :] - centroids[s, :])
 * evaluated in binary32 and rounded once.  The residual is taken against the
 * stored centroid, so a one-member cluster returns expert_out[s] exactly.
 * With LSHMOE_FLAG_NO_RESIDUAL: out[a, :] = expert_out[s, :].
 *
 *   tokens      [T, d]  in   dtype
 *   centroids   [S, d]  in   dtype (as written by lshmoe_compress)
 *   expert_out  [S, d]  in   dtype; E applied to each centroid row, same row order
 *   seg_of      [N]     in   int32, as written by lshmoe_compress
 *   seg_offsets [S+1]   in   int32 or NULL.  When given, one-member clusters skip
 *                            the token and centroid reads (their difference is
 *                            exactly zero); the result is the same either way.
 *   perm [N], num_segments [1]  in  int32 or both NULL, as written by lshmoe_compress.
 *                            When given and the clusters are long on average
 *                            (S / N < 0.65), the rows are produced in cluster order,
 *                            which fetches every cluster's expert-output and centroid
 *                            row once instead of once per member; the result is the
 *                            same either way.
 *   out         [T, k, d] out dtype, assignment order
 *
 * Errors: NULL pointer (seg_offsets excepted; perm and num_segments both or neither); T, d, k <= 0; N >= 2^30
 * (UNSUPPORTED); unknown flag bits (UNSUPPORTED); row size not a multiple of
 * 16 bytes (UNSUPPORTED); launch failure (HIP).
 */
lshmoe_status lshmoe_decompress(const void* tokens, const void* centroids, const void* expert_out,
                                const int32_t* seg_of, const int32_t* seg_offsets,
                                const int32_t* perm, const int32_t* num_segments,
                                int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype, uint32_t flags,
                                void* out, void* stream);

/*
 * Restore fused with the gate-weighted combine of a token's k expert outputs
 * (Eq. 2, with the gate values as weights; Eq. 4 and Eq. 5 for each term):
 *     out[t, :] = sum_{j<k} gate_weight[t][j] *
 *                 (expert_out[s_j, :] + (tokens[t, :] - centroids[s_j, :])),   s_j = seg_of[t*k + j],
 * accumulated in binary32 in the order j = 0..k-1 and rounded once.  It writes
 * one row per token instead of k and reads the token row once.  With
 * LSHMOE_FLAG_NO_RESIDUAL the residual term is dropped.  The paper does not say
 * whether its combine is weighted; pass weights of 1 for the unweighted sum of
 * Eq. 2 as printed.
 *
 *   gate_weight [T, k]  in   binary32 (any values; they are not normalised here)
 *   out         [T, d]  out  dtype
 *   other arguments as for lshmoe_decompress.
 *
 * Errors: as for lshmoe_decompress; NULL gate_weight is LSHMOE_ERR_NULL.
 */
lshmoe_status lshmoe_decompress_combine(const void* tokens, const void* centroids, const void* expert_out,
                                        const int32_t* seg_of, const int32_t* seg_offsets,
                                        const float* gate_weight,
                                        int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype, uint32_t flags,
                                        void* out, void* stream);

/*
 * Backward of lshmoe_decompress / lshmoe_compress with the cluster membership
 * held fixed.  The paper gives no formula for it (Section 3.1 only counts the
 * backward all-to-alls); these two calls are the chain rule applied to the
 * centroid formula of Section 2.3 and to Eq. 4 / Eq. 5:
 *     c_s = (1/n_s) * sum_{a in s} x_a,      Y_a = EC_s + (x_a - c_s).
 * Order of use: lshmoe_decompress_backward turns dL/dY into dL/dEC (S rows, the
 * payload of the backward all-to-all); the experts' backward returns dL/dc for
 * their inputs; lshmoe_compress_backward turns both into dL/dx.
 */

/*
 * Backward of lshmoe_decompress_combine (Eq. 2 with gate weights over Eq. 4 / Eq. 5).  The fused output
 *     out[t, :] = sum_{j<k} w[t][j] * Y[t][j],   Y[t][j] = expert_out[s_j] + (tokens[t] - centroids[s_j])
 * is linear in the weights and in the restored rows, so for grad_out = dL/dout:
 *     grad_gate_weight[t][j] = < grad_out[t, :], Y[t][j] >     binary32; the gradient of the gate's weights
 *     grad_rows[t][j][:]     = w[t][j] * grad_out[t, :]         dtype, rounded once; dL/dY in assignment order
 * The restored rows are formed as in the forward call (from the stored centroids; without the residual term
 * under LSHMOE_FLAG_NO_RESIDUAL) and are not stored.  grad_rows is what lshmoe_decompress_backward and
 * lshmoe_compress_backward take as grad_out, so the three calls in this order give dL/dEC and dL/dx of a layer
 * that uses the fused combine.  The dot products are accumulated in binary32 (each lane its pieces in ascending
 * order, then the lanes pairwise): reproducible bit for bit.
 *
 *   grad_out          [T, d]     in   dtype
 *   gate_weight       [T, k]     in   binary32
 *   grad_gate_weight  [T, k]     out  binary32
 *   grad_rows         [T, k, d]  out  dtype
 *   other arguments as for lshmoe_decompress_combine.
 *
 * Errors: NULL pointer (seg_offsets excepted); T, d, k <= 0; N >= 2^30 or N * d too large for one launch
 * (UNSUPPORTED); unknown flag bits (UNSUPPORTED); row size not a multiple of 16 bytes (UNSUPPORTED); launch failure (HIP).
 */
lshmoe_status lshmoe_decompress_combine_backward(const void* tokens, const void* centroids, const void* expert_out,
                                                 const int32_t* seg_of, const int32_t* seg_offsets,
                                                 const float* gate_weight, const void* grad_out,
                                                 int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype, uint32_t flags,
                                                 float* grad_gate_weight, void* grad_rows, void* stream);

/* Bytes of device scratch lshmoe_decompress_backward needs (host only).  A
 * workspace sized by lshmoe_workspace_bytes for the same T, d, k is also
 * large enough.  Errors: as for lshmoe_workspace_bytes. */
lshmoe_status lshmoe_backward_workspace_bytes(int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype,
                                              size_t* out_bytes);

/*
 * Gradient with respect to the expert outputs: EC_s reaches every member row of
 * cluster s unchanged (Eq. 5), so
 *     grad_expert_out[s, :] = sum_{a in s} grad_out[a, :],
 * members in perm order, accumulated in binary32 (compensated beyond 16
 * members) and rounded once; reproducible bit for bit.
 *
 *   grad_out        [T, k, d] in   dtype; dL/dY in assignment order
 *   perm, seg_offsets, seg_of, num_segments   in, as written by lshmoe_compress
 *   grad_expert_out [N, d]    out  dtype; rows 0..S-1 are written
 *   workspace                 scratch of at least lshmoe_backward_workspace_bytes(...) bytes, 256-byte
 *                             aligned; contents on entry are ignored
 *
 * Errors: NULL pointer; T, d, k <= 0; N >= 2^30 (UNSUPPORTED); row size not a
 * multiple of 16 bytes (UNSUPPORTED); workspace too small or misaligned
 * (WORKSPACE); launch failure (HIP).
 */
lshmoe_status lshmoe_decompress_backward(const void* grad_out, const int32_t* perm, const int32_t* seg_offsets,
                                         const int32_t* seg_of, const int32_t* num_segments,
                                         int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype,
                                         void* grad_expert_out, void* workspace, size_t workspace_bytes,
                                         void* stream);

/*
 * Gradient with respect to the tokens.  The centroid c_s enters the expert
 * (gradient grad_centroids[s]) and, with coefficient -1, every member's Y_a
 * (gradient -grad_expert_out[s] in total), and depends on each member with
 * weight 1/n_s:
 *     grad_tokens[t, :] = sum_{j<k} ( grad_out[a, :] + (grad_centroids[s, :] - grad_expert_out[s, :]) / n_s ),
 *     a = t*k + j,  s = seg_of[a],  n_s = seg_offsets[s+1] - seg_offsets[s],
 * in binary32 in the order j = 0..k-1, rounded once.  For a one-member cluster
 * the term is grad_centroids[s, :] (grad_expert_out[s] is then the row
 * grad_out[a] itself).  With LSHMOE_FLAG_NO_RESIDUAL (forward Y_a = EC_s) the
 * term is grad_centroids[s, :] / n_s, and grad_out and grad_expert_out may be
 * NULL.
 *
 *   grad_out        [T, k, d] in   dtype
 *   grad_centroids  [S, d]    in   dtype; the experts' gradient for their inputs, cluster order
 *   grad_expert_out [S, d]    in   dtype; as written by lshmoe_decompress_backward
 *   seg_of [N], seg_offsets [S+1]  in, as written by lshmoe_compress
 *   grad_tokens     [T, d]    out  dtype
 *
 * Errors: NULL pointer; T, d, k <= 0; N >= 2^30 (UNSUPPORTED); unknown flag
 * bits (UNSUPPORTED); row size not a multiple of 16 bytes (UNSUPPORTED); launch
 * failure (HIP).
 */
lshmoe_status lshmoe_compress_backward(const void* grad_out, const void* grad_centroids, const void* grad_expert_out,
                                       const int32_t* seg_of, const int32_t* seg_offsets,
                                       int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype, uint32_t flags,
                                       void* grad_tokens, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LSHMOE_H */
