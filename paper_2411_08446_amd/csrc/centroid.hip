// Cluster centroids (Section 2.3 centroid formula with 1/n_j; Alg. 1 "Mean"):
// c_s = (1/n_s) * sum of the member rows, members taken in perm order,
// binary32 accumulation, one rounding to the storage type.
//
// HBM-bound gather: reads N token rows (T of them distinct), writes S rows.
// A group of LPR lanes owns one cluster and strides over the 16-byte pieces of
// the row; with rows of 1 KB and more that is a whole wave per cluster, and
// the cluster's offsets and member ids are wave-uniform scalars.  A one-member
// cluster is a plain row copy.  Centroid rows are written with streaming
// stores: nothing in this kernel reads them again.
#include "kernels.h"

namespace lshmoe {

namespace {

constexpr int kPlainSumMax = 16;  // members summed without compensation

template <int LPR> __device__ __forceinline__ int32_t uniform(int32_t v) {
  return LPR == 64 ? __builtin_amdgcn_readfirstlane(v) : v;  // a whole wave shares the value: keep it scalar
}

template <typename DT, int LPR>
__global__ __launch_bounds__(256) void centroid_kernel(
    const char* __restrict__ tokens, const int32_t* __restrict__ perm, const int32_t* __restrict__ seg_offsets,
    const int32_t* __restrict__ num_segments, char* __restrict__ centroids, uint32_t k, uint32_t cpr) {
  constexpr int G = 64 / LPR;  // clusters handled side by side by one wave
  constexpr int E = Piece<DT>::kElems;
  const uint32_t S = (uint32_t)*num_segments;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t s = ((blockIdx.x * 256u + threadIdx.x) >> 6) * G + lane / LPR;
  if (s >= S) return;
  const size_t row_bytes = (size_t)cpr * 16;
  const int32_t lo = uniform<LPR>(seg_offsets[s]), hi = uniform<LPR>(seg_offsets[s + 1]);
  const int32_t n = hi - lo;
  const char* first = tokens + (size_t)((uint32_t)uniform<LPR>(perm[lo]) / k) * row_bytes;
  char* dst = centroids + (size_t)s * row_bytes;
  for (uint32_t c = lane % LPR; c < cpr; c += LPR) {
    const uint4 v0 = load16(first + c * 16);
    if (n == 1) {  // the mean of one row is the row
      store16_stream(dst + c * 16, v0);
      continue;
    }
    float acc[E], x[E];
    Piece<DT>::widen(v0, acc);
    int32_t p = lo + 1;
    if (n <= kPlainSumMax) {
      for (; p + 4 <= hi; p += 4) {
        uint4 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          q[u] = load16(tokens + (size_t)((uint32_t)uniform<LPR>(perm[p + u]) / k) * row_bytes + c * 16);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          Piece<DT>::widen(q[u], x);
#pragma unroll
          for (int i = 0; i < E; ++i) acc[i] += x[i];
        }
      }
      for (; p < hi; ++p) {
        Piece<DT>::widen(load16(tokens + (size_t)((uint32_t)uniform<LPR>(perm[p]) / k) * row_bytes + c * 16), x);
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += x[i];
      }
    } else {
      // long cluster: compensated (Kahan) summation keeps the binary32 sum within
      // a couple of ulps of the exact one however many members there are
      float comp[E];
#pragma unroll
      for (int i = 0; i < E; ++i) comp[i] = 0.0f;
      for (; p < hi; p += 4) {
        uint4 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (p + u < hi) q[u] = load16(tokens + (size_t)((uint32_t)uniform<LPR>(perm[p + u]) / k) * row_bytes + c * 16);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (p + u >= hi) break;
          Piece<DT>::widen(q[u], x);
#pragma unroll
          for (int i = 0; i < E; ++i) {
            const float y = x[i] - comp[i];
            const float t = acc[i] + y;
            comp[i] = (t - acc[i]) - y;
            acc[i] = t;
          }
        }
      }
    }
    const float fn = (float)n;
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] /= fn;
    store16_stream(dst + c * 16, Piece<DT>::narrow(acc));
  }
}

template <typename DT, int LPR>
void launch_lpr(const void* tokens, const int32_t* perm, const int32_t* seg_offsets, const int32_t* num_segments,
                void* centroids, int64_t N, int k, uint32_t cpr, hipStream_t stream) {
  constexpr int G = 64 / LPR;
  const uint64_t waves = ((uint64_t)N + G - 1) / G;  // worst case S == N; surplus waves leave at once
  const uint32_t blocks = (uint32_t)((waves + 3) / 4);
  hipLaunchKernelGGL((centroid_kernel<DT, LPR>), dim3(blocks), dim3(256), 0, stream, (const char*)tokens, perm,
                     seg_offsets, num_segments, (char*)centroids, (uint32_t)k, cpr);
}

template <typename DT>
void launch_typed(const void* tokens, const int32_t* perm, const int32_t* seg_offsets, const int32_t* num_segments,
                  void* centroids, int64_t N, int k, uint32_t cpr, hipStream_t stream) {
  if (cpr > 16) launch_lpr<DT, 64>(tokens, perm, seg_offsets, num_segments, centroids, N, k, cpr, stream);
  else if (cpr > 4) launch_lpr<DT, 16>(tokens, perm, seg_offsets, num_segments, centroids, N, k, cpr, stream);
  else launch_lpr<DT, 4>(tokens, perm, seg_offsets, num_segments, centroids, N, k, cpr, stream);
}

}  // namespace

hipError_t launch_centroid(const void* tokens, const int32_t* perm, const int32_t* seg_offsets,
                           const int32_t* num_segments, void* centroids, int64_t N, int k, int d, bool bf16,
                           hipStream_t stream) {
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  if (bf16) launch_typed<BF16>(tokens, perm, seg_offsets, num_segments, centroids, N, k, cpr, stream);
  else launch_typed<F32>(tokens, perm, seg_offsets, num_segments, centroids, N, k, cpr, stream);
  return hipGetLastError();
}

}  // namespace lshmoe
