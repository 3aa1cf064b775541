// Cluster centroids (Section 2.3 centroid formula with 1/n_j; Alg. 1 "Mean"):
// c_s = (1/n_s) * sum of the member rows, members taken in perm order,
// binary32 accumulation, one rounding to the storage type.
//
// One thread owns one 16-byte chunk of one centroid row and walks the
// cluster's members; rows are gathered through perm.  HBM-bound: reads N rows
// (T of them distinct), writes S rows.
#include "kernels.h"

namespace lshmoe {

constexpr int kPlainSumMax = 16;  // members summed without compensation

template <typename DT>
__global__ __launch_bounds__(256) void centroid_kernel(
    const char* __restrict__ tokens, const int32_t* __restrict__ perm, const int32_t* __restrict__ seg_offsets,
    const int32_t* __restrict__ num_segments, char* __restrict__ centroids, uint32_t k, uint32_t cpr) {
  const uint32_t S = (uint32_t)*num_segments;
  const uint32_t g = blockIdx.x * 256u + threadIdx.x;
  const uint32_t s = g / cpr;
  const uint32_t c = g - s * cpr;
  if (s >= S) return;
  const size_t row_bytes = (size_t)cpr * 16;
  const int32_t lo = seg_offsets[s], hi = seg_offsets[s + 1];
  constexpr int E = Chunk<DT>::kElems;
  float acc[E];
#pragma unroll
  for (int i = 0; i < E; ++i) acc[i] = 0.0f;
  int32_t p = lo;
  if (hi - lo <= kPlainSumMax) {
    for (; p + 4 <= hi; p += 4) {
      Chunk<DT> x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u].load(tokens + (size_t)((uint32_t)perm[p + u] / k) * row_bytes, c);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += x[u].v[i];
    }
    for (; p < hi; ++p) {
      Chunk<DT> x;
      x.load(tokens + (size_t)((uint32_t)perm[p] / k) * row_bytes, c);
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] += x.v[i];
    }
  } else {
    // long cluster: compensated (Kahan) summation keeps the binary32 sum within
    // a couple of ulps of the exact one however many members there are
    float comp[E];
#pragma unroll
    for (int i = 0; i < E; ++i) comp[i] = 0.0f;
    for (; p < hi; p += 4) {
      Chunk<DT> x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (p + u < hi) x[u].load(tokens + (size_t)((uint32_t)perm[p + u] / k) * row_bytes, c);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (p + u >= hi) break;
#pragma unroll
        for (int i = 0; i < E; ++i) {
          const float y = x[u].v[i] - comp[i];
          const float t = acc[i] + y;
          comp[i] = (t - acc[i]) - y;
          acc[i] = t;
        }
      }
    }
  }
  const float n = (float)(hi - lo);
  Chunk<DT> out;
#pragma unroll
  for (int i = 0; i < E; ++i) out.v[i] = acc[i] / n;
  out.store(centroids + (size_t)s * row_bytes, c);
}

hipError_t launch_centroid(const void* tokens, const int32_t* perm, const int32_t* seg_offsets,
                           const int32_t* num_segments, void* centroids, int64_t N, int k, int d, bool bf16,
                           hipStream_t stream) {
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  const uint64_t threads = (uint64_t)N * cpr;  // worst case S == N; surplus threads leave at once
  if (threads > 0xffffff00ull) return hipErrorInvalidValue;
  const uint32_t blocks = (uint32_t)((threads + 255) / 256);
  if (bf16)
    hipLaunchKernelGGL(centroid_kernel<BF16>, dim3(blocks), dim3(256), 0, stream, (const char*)tokens, perm,
                       seg_offsets, num_segments, (char*)centroids, (uint32_t)k, cpr);
  else
    hipLaunchKernelGGL(centroid_kernel<F32>, dim3(blocks), dim3(256), 0, stream, (const char*)tokens, perm,
                       seg_offsets, num_segments, (char*)centroids, (uint32_t)k, cpr);
  return hipGetLastError();
}

}  // namespace lshmoe
