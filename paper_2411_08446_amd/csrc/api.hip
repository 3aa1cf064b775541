// C ABI of the library: argument checks on the host, then kernel launches.
// Every check runs before the first HIP call, so bad arguments are reported
// the same way on a machine without a GPU.
#include <stdarg.h>
#include <stdio.h>

#include <atomic>

#include "../../include/lshmoe.h"
#include "kernels.h"

namespace {

thread_local char g_err[512] = "";

lshmoe_status fail(lshmoe_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return st;
}

lshmoe_status ok() {
  g_err[0] = '\0';
  return LSHMOE_OK;
}

lshmoe_status hip_fail(const char* what, hipError_t e) {
  return fail(LSHMOE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool dtype_ok(int dt) { return dt == LSHMOE_F32 || dt == LSHMOE_BF16; }
size_t item_size(int dt) { return dt == LSHMOE_BF16 ? 2 : 4; }

// (2r)^L < 2^63 ?
bool bucket_space_ok(int L, int r) {
  unsigned __int128 nb = 1;
  for (int l = 0; l < L; ++l) {
    nb *= (unsigned __int128)(2 * (uint64_t)r);
    if (nb >= ((unsigned __int128)1 << 63)) return false;
  }
  return true;
}

constexpr int64_t kMaxAssignments = (int64_t)1 << 30;

lshmoe_status check_row(int d, int dt) {
  if (!dtype_ok(dt)) return fail(LSHMOE_ERR_UNSUPPORTED, "unknown dtype %d", dt);
  if (((size_t)d * item_size(dt)) % 16 != 0)
    return fail(LSHMOE_ERR_UNSUPPORTED, "row size d*sizeof(element) = %zu bytes is not a multiple of 16",
                (size_t)d * item_size(dt));
  return LSHMOE_OK;
}

lshmoe_status check_hash_params(int L, int r) {
  if (L <= 0 || r <= 0) return fail(LSHMOE_ERR_SHAPE, "L and r must be positive (L=%d, r=%d)", L, r);
  if (r < 2) return fail(LSHMOE_ERR_UNSUPPORTED, "r must be at least 2 (r=%d)", r);
  if (!bucket_space_ok(L, r)) return fail(LSHMOE_ERR_UNSUPPORTED, "(2r)^L does not fit below 2^63 (L=%d, r=%d)", L, r);
  return LSHMOE_OK;
}

lshmoe_status check_compress_shape(int64_t T, int d, int k, int E, int L, int r, int dt, lshmoe::GroupPlan* plan) {
  if (T <= 0 || d <= 0 || k <= 0 || E <= 0)
    return fail(LSHMOE_ERR_SHAPE, "T, d, k, E must be positive (T=%lld, d=%d, k=%d, E=%d)", (long long)T, d, k, E);
  if (k > E) return fail(LSHMOE_ERR_SHAPE, "k=%d experts per token exceeds E=%d experts", k, E);
  if (lshmoe_status st = check_hash_params(L, r)) return st;
  if (lshmoe_status st = check_row(d, dt)) return st;
  if (T >= kMaxAssignments || T * (int64_t)k >= kMaxAssignments)
    return fail(LSHMOE_ERR_UNSUPPORTED, "N = T*k = %lld assignments; the limit is 2^30 - 1", (long long)(T * (int64_t)k));
  if ((uint64_t)T * (uint64_t)k * ((size_t)d * item_size(dt) / 16) > 0xffffff00ull)
    return fail(LSHMOE_ERR_UNSUPPORTED, "N*d is too large for one launch");
  if (!lshmoe::plan_group(T, d, k, E, L, r, plan))
    return fail(LSHMOE_ERR_UNSUPPORTED, "expert bits + bucket bits exceed 64 (E=%d, L=%d, r=%d)", E, L, r);
  return LSHMOE_OK;
}

// T, d, k and the row size of an entry point that moves [N, d] rows.
lshmoe_status check_rows_shape(int64_t T, int d, int k, int dt) {
  if (T <= 0 || d <= 0 || k <= 0)
    return fail(LSHMOE_ERR_SHAPE, "T, d, k must be positive (T=%lld, d=%d, k=%d)", (long long)T, d, k);
  if (lshmoe_status st = check_row(d, dt)) return st;
  if (T >= kMaxAssignments || T * (int64_t)k >= kMaxAssignments)
    return fail(LSHMOE_ERR_UNSUPPORTED, "N = T*k = %lld assignments; the limit is 2^30 - 1", (long long)(T * (int64_t)k));
  if ((uint64_t)T * (uint64_t)k * ((size_t)d * item_size(dt) / 16) > 0xffffff00ull)
    return fail(LSHMOE_ERR_UNSUPPORTED, "N*d is too large for one launch");
  return LSHMOE_OK;
}

// Scratch of lshmoe_compress_static: device memory that belongs to the library image, so that the call needs no
// allocation.  Every GPU the library runs on holds its own copy until the process ends.  In host code the name is
// only a handle; the device address is looked up once per device and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = LSHMOE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
lshmoe_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail("hipGetDevice", e);
  if (dev < 0 || dev >= kMaxDevices) return fail(LSHMOE_ERR_UNSUPPORTED, "device ordinal %d; the limit is %d", dev, kMaxDevices - 1);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail("hipGetSymbolAddress(scratch)", e);
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
  }
  *out = p;
  return LSHMOE_OK;
}

}  // namespace

extern "C" {

const char* lshmoe_status_string(int status) {
  switch (status) {
    case LSHMOE_OK: return "LSHMOE_OK";
    case LSHMOE_ERR_NULL: return "LSHMOE_ERR_NULL";
    case LSHMOE_ERR_SHAPE: return "LSHMOE_ERR_SHAPE";
    case LSHMOE_ERR_UNSUPPORTED: return "LSHMOE_ERR_UNSUPPORTED";
    case LSHMOE_ERR_WORKSPACE: return "LSHMOE_ERR_WORKSPACE";
    case LSHMOE_ERR_HIP: return "LSHMOE_ERR_HIP";
    default: return "LSHMOE_ERR_UNKNOWN";
  }
}

const char* lshmoe_last_error(void) { return g_err; }

int lshmoe_abi_version(void) { return 6; }

lshmoe_status lshmoe_workspace_bytes(int64_t T, int32_t d, int32_t k, int32_t E, int32_t L, int32_t r,
                                     lshmoe_dtype dtype, size_t* out_bytes) {
  if (!out_bytes) return fail(LSHMOE_ERR_NULL, "out_bytes is NULL");
  lshmoe::GroupPlan plan;
  if (lshmoe_status st = check_compress_shape(T, d, k, E, L, r, (int)dtype, &plan)) return st;
  *out_bytes = plan.total_bytes;
  return ok();
}

lshmoe_status lshmoe_hash(const void* tokens, const void* rot, int64_t T, int32_t d, int32_t L, int32_t r,
                          lshmoe_dtype dtype, uint64_t* bucket, void* stream) {
  if (!tokens || !rot || !bucket) return fail(LSHMOE_ERR_NULL, "tokens, rot and bucket must be non-NULL");
  if (T <= 0 || d <= 0) return fail(LSHMOE_ERR_SHAPE, "T and d must be positive (T=%lld, d=%d)", (long long)T, d);
  if (lshmoe_status st = check_hash_params(L, r)) return st;
  if (lshmoe_status st = check_row(d, (int)dtype)) return st;
  if (T >= kMaxAssignments) return fail(LSHMOE_ERR_UNSUPPORTED, "T = %lld tokens; the limit is 2^30 - 1", (long long)T);
  if (r > 256) return fail(LSHMOE_ERR_UNSUPPORTED, "r = %d rotated dimensions per hash; the limit is 256", r);
  hipError_t e = lshmoe::launch_hash(tokens, rot, T, d, L, r, dtype == LSHMOE_BF16, bucket, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("hash launch", e);
  return ok();
}

lshmoe_status lshmoe_hash_sphere(const void* tokens, const void* pivots, const float* radius_sq, int64_t T, int32_t d,
                                 int32_t B, lshmoe_dtype dtype, uint64_t* bucket, void* stream) {
  if (!tokens || !pivots || !radius_sq || !bucket)
    return fail(LSHMOE_ERR_NULL, "tokens, pivots, radius_sq and bucket must be non-NULL");
  if (T <= 0 || d <= 0 || B <= 0) return fail(LSHMOE_ERR_SHAPE, "T, d and B must be positive (T=%lld, d=%d, B=%d)", (long long)T, d, B);
  if (B > 63) return fail(LSHMOE_ERR_UNSUPPORTED, "B = %d spheres; the code is one bit per sphere and the limit is 63", B);
  if (lshmoe_status st = check_row(d, (int)dtype)) return st;
  if (T >= kMaxAssignments) return fail(LSHMOE_ERR_UNSUPPORTED, "T = %lld tokens; the limit is 2^30 - 1", (long long)T);
  hipError_t e = lshmoe::launch_hash_sphere(tokens, pivots, radius_sq, T, d, B, dtype == LSHMOE_BF16, bucket,
                                            (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("spherical hash launch", e);
  return ok();
}

lshmoe_status lshmoe_hash_gate(const void* tokens, const void* rot, const void* gate_w, int64_t T, int32_t d, int32_t L,
                               int32_t r, int32_t E, lshmoe_dtype dtype, uint64_t* bucket, float* logits, void* stream) {
  if (!tokens || !rot || !gate_w || !bucket || !logits)
    return fail(LSHMOE_ERR_NULL, "tokens, rot, gate_w, bucket and logits must be non-NULL");
  if (T <= 0 || d <= 0 || E <= 0)
    return fail(LSHMOE_ERR_SHAPE, "T, d and E must be positive (T=%lld, d=%d, E=%d)", (long long)T, d, E);
  if (lshmoe_status st = check_hash_params(L, r)) return st;
  if (lshmoe_status st = check_row(d, (int)dtype)) return st;
  if (T >= kMaxAssignments) return fail(LSHMOE_ERR_UNSUPPORTED, "T = %lld tokens; the limit is 2^30 - 1", (long long)T);
  if (r > 256) return fail(LSHMOE_ERR_UNSUPPORTED, "r = %d rotated dimensions per hash; the limit is 256", r);
  if (!lshmoe::hash_gate_supported(d, r, E, dtype == LSHMOE_BF16))
    return fail(LSHMOE_ERR_UNSUPPORTED,
                "the fused gate needs r a multiple of 8, rows of whole 512-byte blocks and E <= 128 (r=%d, d=%d, E=%d)", r,
                d, E);
  hipError_t e = lshmoe::launch_hash_gate(tokens, rot, gate_w, T, d, L, r, E, dtype == LSHMOE_BF16, bucket, logits,
                                          (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("hash + gate launch", e);
  return ok();
}

lshmoe_status lshmoe_compress(const void* tokens, const int32_t* expert, const uint64_t* bucket, int64_t T, int32_t d,
                              int32_t k, int32_t E, int32_t L, int32_t r, lshmoe_dtype dtype, void* centroids,
                              int32_t* seg_offsets, int32_t* seg_expert, int32_t* expert_offsets, int32_t* perm,
                              int32_t* seg_of, int32_t* num_segments, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!tokens || !expert || !bucket || !centroids || !seg_offsets || !seg_expert || !expert_offsets || !perm ||
      !seg_of || !num_segments)
    return fail(LSHMOE_ERR_NULL, "an input or output pointer is NULL");
  lshmoe::GroupPlan plan;
  if (lshmoe_status st = check_compress_shape(T, d, k, E, L, r, (int)dtype, &plan)) return st;
  if (!workspace) return fail(LSHMOE_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", plan.total_bytes);
  if (((uintptr_t)workspace & 255u) != 0) return fail(LSHMOE_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < plan.total_bytes)
    return fail(LSHMOE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, plan.total_bytes);
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = lshmoe::launch_group(plan, expert, bucket, k, E, seg_offsets, seg_expert, expert_offsets, perm, seg_of,
                                      num_segments, (char*)workspace, s);
  if (e != hipSuccess) return hip_fail("group launch", e);
  e = lshmoe::launch_centroid(tokens, perm, seg_offsets, seg_of, num_segments, centroids,
                              (float*)((char*)workspace + plan.off_partial),
                              (uint32_t*)((char*)workspace + plan.off_counters), plan.N, k, d, dtype == LSHMOE_BF16,
                              /*mean=*/true, s);
  if (e != hipSuccess) return hip_fail("centroid launch", e);
  return ok();
}

lshmoe_status lshmoe_compress_static(const void* tokens, const int32_t* expert, const uint64_t* bucket, int64_t T,
                                     int32_t d, int32_t k, int32_t E, int32_t L, int32_t r, lshmoe_dtype dtype,
                                     void* centroids, int32_t* seg_offsets, int32_t* seg_expert, int32_t* expert_offsets,
                                     int32_t* perm, int32_t* seg_of, int32_t* num_segments, void* stream) {
  if (!tokens || !expert || !bucket || !centroids || !seg_offsets || !seg_expert || !expert_offsets || !perm ||
      !seg_of || !num_segments)
    return fail(LSHMOE_ERR_NULL, "an input or output pointer is NULL");
  lshmoe::GroupPlan plan;
  if (lshmoe_status st = check_compress_shape(T, d, k, E, L, r, (int)dtype, &plan)) return st;
  if (plan.total_bytes > kStaticScratchBytes)
    return fail(LSHMOE_ERR_WORKSPACE,
                "these sizes need %zu bytes of scratch; the built-in scratch of lshmoe_compress_static holds %zu "
                "(use lshmoe_compress with a workspace of the caller's)", plan.total_bytes, kStaticScratchBytes);
  void* ws = nullptr;
  if (lshmoe_status st = static_scratch(&ws)) return st;
  return lshmoe_compress(tokens, expert, bucket, T, d, k, E, L, r, dtype, centroids, seg_offsets, seg_expert,
                         expert_offsets, perm, seg_of, num_segments, ws, kStaticScratchBytes, stream);
}

lshmoe_status lshmoe_decompress(const void* tokens, const void* centroids, const void* expert_out,
                                const int32_t* seg_of, const int32_t* seg_offsets, const int32_t* perm,
                                const int32_t* num_segments, int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype,
                                uint32_t flags, void* out, void* stream) {
  if (!tokens || !centroids || !expert_out || !seg_of || !out)
    return fail(LSHMOE_ERR_NULL, "an input or output pointer is NULL");
  if (T <= 0 || d <= 0 || k <= 0)
    return fail(LSHMOE_ERR_SHAPE, "T, d, k must be positive (T=%lld, d=%d, k=%d)", (long long)T, d, k);
  if (lshmoe_status st = check_row(d, (int)dtype)) return st;
  if (flags & ~(uint32_t)LSHMOE_FLAG_NO_RESIDUAL) return fail(LSHMOE_ERR_UNSUPPORTED, "unknown flag bits 0x%x", flags);
  if (T >= kMaxAssignments || T * (int64_t)k >= kMaxAssignments)
    return fail(LSHMOE_ERR_UNSUPPORTED, "N = T*k = %lld assignments; the limit is 2^30 - 1", (long long)(T * (int64_t)k));
  if ((uint64_t)T * (uint64_t)k * ((size_t)d * item_size((int)dtype) / 16) > 0xffffff00ull)
    return fail(LSHMOE_ERR_UNSUPPORTED, "N*d is too large for one launch");
  if ((perm == nullptr) != (num_segments == nullptr))
    return fail(LSHMOE_ERR_NULL, "perm and num_segments are given together or not at all");
  hipError_t e = lshmoe::launch_restore(tokens, centroids, expert_out, seg_of, seg_offsets, perm, num_segments, out,
                                        T * (int64_t)k, k, d, dtype == LSHMOE_BF16, flags, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("restore launch", e);
  return ok();
}

lshmoe_status lshmoe_decompress_combine(const void* tokens, const void* centroids, const void* expert_out,
                                        const int32_t* seg_of, const int32_t* seg_offsets, const float* gate_weight,
                                        int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype, uint32_t flags, void* out,
                                        void* stream) {
  if (!tokens || !centroids || !expert_out || !seg_of || !gate_weight || !out)
    return fail(LSHMOE_ERR_NULL, "an input or output pointer is NULL");
  if (T <= 0 || d <= 0 || k <= 0)
    return fail(LSHMOE_ERR_SHAPE, "T, d, k must be positive (T=%lld, d=%d, k=%d)", (long long)T, d, k);
  if (lshmoe_status st = check_row(d, (int)dtype)) return st;
  if (flags & ~(uint32_t)LSHMOE_FLAG_NO_RESIDUAL) return fail(LSHMOE_ERR_UNSUPPORTED, "unknown flag bits 0x%x", flags);
  if (T >= kMaxAssignments || T * (int64_t)k >= kMaxAssignments)
    return fail(LSHMOE_ERR_UNSUPPORTED, "N = T*k = %lld assignments; the limit is 2^30 - 1", (long long)(T * (int64_t)k));
  hipError_t e = lshmoe::launch_restore_combine(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, out, T,
                                                k, d, dtype == LSHMOE_BF16, flags, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("restore-combine launch", e);
  return ok();
}

lshmoe_status lshmoe_decompress_combine_backward(const void* tokens, const void* centroids, const void* expert_out,
                                                 const int32_t* seg_of, const int32_t* seg_offsets,
                                                 const float* gate_weight, const void* grad_out, int64_t T, int32_t d,
                                                 int32_t k, lshmoe_dtype dtype, uint32_t flags, float* grad_gate_weight,
                                                 void* grad_rows, void* stream) {
  if (!tokens || !centroids || !expert_out || !seg_of || !gate_weight || !grad_out || !grad_gate_weight || !grad_rows)
    return fail(LSHMOE_ERR_NULL, "an input or output pointer is NULL");
  if (flags & ~(uint32_t)LSHMOE_FLAG_NO_RESIDUAL) return fail(LSHMOE_ERR_UNSUPPORTED, "unknown flag bits 0x%x", flags);
  if (lshmoe_status st = check_rows_shape(T, d, k, (int)dtype)) return st;
  hipError_t e = lshmoe::launch_combine_backward(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, grad_out,
                                                 grad_gate_weight, grad_rows, T, k, d, dtype == LSHMOE_BF16, flags,
                                                 (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("combine backward launch", e);
  return ok();
}

lshmoe_status lshmoe_backward_workspace_bytes(int64_t T, int32_t d, int32_t k, lshmoe_dtype dtype, size_t* out_bytes) {
  if (!out_bytes) return fail(LSHMOE_ERR_NULL, "out_bytes is NULL");
  if (lshmoe_status st = check_rows_shape(T, d, k, (int)dtype)) return st;
  *out_bytes = lshmoe::plan_backward(T * (int64_t)k, d).total_bytes;
  return ok();
}

lshmoe_status lshmoe_decompress_backward(const void* grad_out, const int32_t* perm, const int32_t* seg_offsets,
                                         const int32_t* seg_of, const int32_t* num_segments, int64_t T, int32_t d,
                                         int32_t k, lshmoe_dtype dtype, void* grad_expert_out, void* workspace,
                                         size_t workspace_bytes, void* stream) {
  if (!grad_out || !perm || !seg_offsets || !seg_of || !num_segments || !grad_expert_out)
    return fail(LSHMOE_ERR_NULL, "an input or output pointer is NULL");
  if (lshmoe_status st = check_rows_shape(T, d, k, (int)dtype)) return st;
  const int64_t N = T * (int64_t)k;
  const lshmoe::BackwardPlan plan = lshmoe::plan_backward(N, d);
  if (!workspace) return fail(LSHMOE_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", plan.total_bytes);
  if (((uintptr_t)workspace & 255u) != 0) return fail(LSHMOE_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (workspace_bytes < plan.total_bytes)
    return fail(LSHMOE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, plan.total_bytes);
  hipStream_t s = (hipStream_t)stream;
  uint32_t* counters = (uint32_t*)((char*)workspace + plan.off_counters);
  hipError_t e = lshmoe::launch_clear_counters(counters, plan.windows, s);
  if (e != hipSuccess) return hip_fail("counter clear launch", e);
  // a segment sum over the rows of grad_out: row of sorted position p is grad_out[perm[p]]
  e = lshmoe::launch_centroid(grad_out, perm, seg_offsets, seg_of, num_segments, grad_expert_out,
                              (float*)((char*)workspace + plan.off_partial), counters, N, /*k=*/1, d,
                              dtype == LSHMOE_BF16, /*mean=*/false, s);
  if (e != hipSuccess) return hip_fail("segment sum launch", e);
  return ok();
}

lshmoe_status lshmoe_compress_backward(const void* grad_out, const void* grad_centroids, const void* grad_expert_out,
                                       const int32_t* seg_of, const int32_t* seg_offsets, int64_t T, int32_t d,
                                       int32_t k, lshmoe_dtype dtype, uint32_t flags, void* grad_tokens, void* stream) {
  if (!grad_centroids || !seg_of || !seg_offsets || !grad_tokens)
    return fail(LSHMOE_ERR_NULL, "an input or output pointer is NULL");
  if (flags & ~(uint32_t)LSHMOE_FLAG_NO_RESIDUAL) return fail(LSHMOE_ERR_UNSUPPORTED, "unknown flag bits 0x%x", flags);
  if (!(flags & LSHMOE_FLAG_NO_RESIDUAL) && (!grad_out || !grad_expert_out))
    return fail(LSHMOE_ERR_NULL, "grad_out and grad_expert_out are required unless LSHMOE_FLAG_NO_RESIDUAL is set");
  if (lshmoe_status st = check_rows_shape(T, d, k, (int)dtype)) return st;
  hipError_t e = lshmoe::launch_grad_tokens(grad_out, grad_centroids, grad_expert_out, seg_of, seg_offsets, grad_tokens,
                                            T, k, d, dtype == LSHMOE_BF16, flags, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("token gradient launch", e);
  return ok();
}

}  // extern "C"
