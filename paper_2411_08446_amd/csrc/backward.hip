// Backward of the centroid and restore steps, cluster membership held fixed
// (the paper gives no formula; this is the chain rule for
//   c_s = (1/n_s) sum_{a in s} x_a,   Y_a = EC_s + (x_a - c_s)).
//
// dL/dEC_s = sum_{a in s} dL/dY_a is a segment sum over the rows of dL/dY: the
// centroid kernel with the division left out (launch_centroid, mean = false).
// This file holds the other half: per token,
//   dL/dx_t = sum_j ( dL/dY_a + (h_s - G_s) / n_s ),  a = t*k + j, s = seg_of[a],
// with h_s the expert's gradient for its input c_s and G_s the stored segment
// sum.  HBM-bound gather like the restore; for a one-member cluster G_s is the
// row dL/dY_a itself, so the term is h_s and two of the three reads are skipped.
#include "kernels.h"

namespace lshmoe {

namespace {

template <int LPR> __device__ __forceinline__ int32_t uniform(int32_t v) {
  return LPR == 64 ? __builtin_amdgcn_readfirstlane(v) : v;
}

template <typename DT, int LPR>
__global__ __launch_bounds__(256) void grad_tokens_kernel(
    const char* __restrict__ grad_out, const char* __restrict__ grad_centroids,
    const char* __restrict__ grad_expert_out, const int32_t* __restrict__ seg_of,
    const int32_t* __restrict__ seg_offsets, char* __restrict__ grad_tokens, uint32_t T, uint32_t k, uint32_t cpr,
    uint32_t flags) {
  constexpr int G = 64 / LPR;
  constexpr int E = Piece<DT>::kElems;
  const uint32_t lane = threadIdx.x & 63;
  const uint64_t wave64 = linear_block() * 4u + (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (wave64 * G >= T) return;
  const uint32_t t = (uint32_t)(wave64 * G) + lane / LPR;   // below T + 64: 32 bits are enough
  if (t >= T) return;
  const size_t row_bytes = (size_t)cpr * 16;
  const bool no_res = (flags & 1u) != 0;
  for (uint32_t c = lane % LPR; c < cpr; c += LPR) {
    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.0f;
    for (uint32_t j = 0; j < k; ++j) {
      const uint32_t a = t * k + j;
      const int32_t s = uniform<LPR>(seg_of[a]);
      const int32_t n = uniform<LPR>(seg_offsets[s + 1]) - uniform<LPR>(seg_offsets[s]);
      float h[E];
      Piece<DT>::widen(load16(grad_centroids + (size_t)s * row_bytes + c * 16), h);
      if (n == 1) {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += h[i];
      } else if (no_res) {
        const float fn = (float)n;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += h[i] / fn;
      } else {
        float g[E], gs[E];
        Piece<DT>::widen(load16(grad_out + (size_t)a * row_bytes + c * 16), g);
        Piece<DT>::widen(load16(grad_expert_out + (size_t)s * row_bytes + c * 16), gs);
        const float fn = (float)n;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += g[i] + (h[i] - gs[i]) / fn;
      }
    }
    store16_stream(grad_tokens + (size_t)t * row_bytes + c * 16, Piece<DT>::narrow(acc));
  }
}

template <typename DT, int LPR>
void launch_lpr(const void* grad_out, const void* grad_centroids, const void* grad_expert_out, const int32_t* seg_of,
                const int32_t* seg_offsets, void* grad_tokens, int64_t T, int k, uint32_t cpr, uint32_t flags,
                hipStream_t stream) {
  constexpr int G = 64 / LPR;
  const uint64_t waves = ((uint64_t)T + G - 1) / G;
  const uint32_t blocks = (uint32_t)((waves + 3) / 4);
  hipLaunchKernelGGL((grad_tokens_kernel<DT, LPR>), grid_of_blocks(blocks), dim3(256), 0, stream, (const char*)grad_out,
                     (const char*)grad_centroids, (const char*)grad_expert_out, seg_of, seg_offsets,
                     (char*)grad_tokens, (uint32_t)T, (uint32_t)k, cpr, flags);
}

template <typename DT>
void launch_typed(const void* grad_out, const void* grad_centroids, const void* grad_expert_out, const int32_t* seg_of,
                  const int32_t* seg_offsets, void* grad_tokens, int64_t T, int k, uint32_t cpr, uint32_t flags,
                  hipStream_t stream) {
  if (cpr > 16)
    launch_lpr<DT, 64>(grad_out, grad_centroids, grad_expert_out, seg_of, seg_offsets, grad_tokens, T, k, cpr, flags, stream);
  else if (cpr > 4)
    launch_lpr<DT, 16>(grad_out, grad_centroids, grad_expert_out, seg_of, seg_offsets, grad_tokens, T, k, cpr, flags, stream);
  else
    launch_lpr<DT, 4>(grad_out, grad_centroids, grad_expert_out, seg_of, seg_offsets, grad_tokens, T, k, cpr, flags, stream);
}

__global__ __launch_bounds__(256) void clear_u32_kernel(uint32_t* __restrict__ p, uint32_t n) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace

hipError_t launch_grad_tokens(const void* grad_out, const void* grad_centroids, const void* grad_expert_out,
                              const int32_t* seg_of, const int32_t* seg_offsets, void* grad_tokens, int64_t T, int k,
                              int d, bool bf16, uint32_t flags, hipStream_t stream) {
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  if (bf16)
    launch_typed<BF16>(grad_out, grad_centroids, grad_expert_out, seg_of, seg_offsets, grad_tokens, T, k, cpr, flags, stream);
  else
    launch_typed<F32>(grad_out, grad_centroids, grad_expert_out, seg_of, seg_offsets, grad_tokens, T, k, cpr, flags, stream);
  return hipGetLastError();
}

BackwardPlan plan_backward(int64_t N, int d) {
  BackwardPlan p{};
  p.windows = 2 * (size_t)((N + kCentroidWindow - 1) / kCentroidWindow);
  p.off_partial = 0;
  size_t off = (p.windows * (size_t)d * 4 + 255) & ~(size_t)255;
  p.off_counters = off;
  off = (off + p.windows * 4 + 255) & ~(size_t)255;
  p.total_bytes = off;
  return p;
}

hipError_t launch_clear_counters(uint32_t* counters, size_t n, hipStream_t stream) {
  hipLaunchKernelGGL(clear_u32_kernel, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, stream, counters, (uint32_t)n);
  return hipGetLastError();
}

}  // namespace lshmoe
