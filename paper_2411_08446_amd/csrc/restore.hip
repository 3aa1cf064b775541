// Restore with residual compensation (Eq. 4 and Eq. 5): one 16-byte chunk of
// one output row per thread and unroll step.  HBM-bound gather: per output
// row it reads the token row, the centroid row and the expert-output row and
// writes one row; one-member clusters read only the expert-output row.
#include "kernels.h"

namespace lshmoe {

template <typename DT, int UNROLL>
__global__ __launch_bounds__(256) void restore_kernel(
    const char* __restrict__ tokens, const char* __restrict__ centroids, const char* __restrict__ expert_out,
    const int32_t* __restrict__ seg_of, const int32_t* __restrict__ seg_offsets, char* __restrict__ out,
    uint32_t N, uint32_t k, uint32_t cpr, uint32_t rows_per_sweep, uint32_t flags) {
  const uint32_t g = blockIdx.x * 256u + threadIdx.x;
  const uint32_t a0 = g / cpr;
  const uint32_t c = g - a0 * cpr;
  if (a0 >= rows_per_sweep) return;
  const size_t row_bytes = (size_t)cpr * 16;
  const bool no_res = (flags & 1u) != 0;

  int32_t s[UNROLL];
  bool live[UNROLL], full[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const uint32_t a = a0 + u * rows_per_sweep;
    live[u] = a < N;
    s[u] = live[u] ? seg_of[a] : 0;
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    full[u] = live[u] && !no_res;
    if (full[u] && seg_offsets != nullptr) full[u] = (seg_offsets[s[u] + 1] - seg_offsets[s[u]]) != 1;
  }
  Chunk<DT> ec[UNROLL], x[UNROLL], cc[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    if (live[u]) ec[u].load(expert_out + (size_t)s[u] * row_bytes, c);
    if (full[u]) {
      const uint32_t a = a0 + u * rows_per_sweep;
      x[u].load(tokens + (size_t)(a / k) * row_bytes, c);
      cc[u].load(centroids + (size_t)s[u] * row_bytes, c);
    }
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    if (!live[u]) continue;
    const uint32_t a = a0 + u * rows_per_sweep;
    Chunk<DT> y;
    if (full[u]) {
#pragma unroll
      for (int i = 0; i < Chunk<DT>::kElems; ++i) y.v[i] = ec[u].v[i] + (x[u].v[i] - cc[u].v[i]);
    } else if (no_res) {
#pragma unroll
      for (int i = 0; i < Chunk<DT>::kElems; ++i) y.v[i] = ec[u].v[i];
    } else {
      // x == c bit for bit: the residual is +0, and e + (+0) maps -0 to +0
#pragma unroll
      for (int i = 0; i < Chunk<DT>::kElems; ++i) y.v[i] = ec[u].v[i] + 0.0f;
    }
    y.store(out + (size_t)a * row_bytes, c);
  }
}

hipError_t launch_restore(const void* tokens, const void* centroids, const void* expert_out,
                          const int32_t* seg_of, const int32_t* seg_offsets, void* out,
                          int64_t N, int k, int d, bool bf16, uint32_t flags, hipStream_t stream) {
  constexpr int UNROLL = 4;
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  const uint32_t rows_per_sweep = (uint32_t)((N + UNROLL - 1) / UNROLL);
  const uint64_t threads = (uint64_t)rows_per_sweep * cpr;
  if (threads > 0xffffff00ull) return hipErrorInvalidValue;
  const uint32_t blocks = (uint32_t)((threads + 255) / 256);
  auto t = (const char*)tokens;
  auto c = (const char*)centroids;
  auto e = (const char*)expert_out;
  if (bf16)
    hipLaunchKernelGGL((restore_kernel<BF16, UNROLL>), dim3(blocks), dim3(256), 0, stream, t, c, e, seg_of,
                       seg_offsets, (char*)out, (uint32_t)N, (uint32_t)k, cpr, rows_per_sweep, flags);
  else
    hipLaunchKernelGGL((restore_kernel<F32, UNROLL>), dim3(blocks), dim3(256), 0, stream, t, c, e, seg_of,
                       seg_offsets, (char*)out, (uint32_t)N, (uint32_t)k, cpr, rows_per_sweep, flags);
  return hipGetLastError();
}

}  // namespace lshmoe
