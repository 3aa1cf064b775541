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

// Backward of the restore fused with the gate-weighted combine,
//     out[t] = sum_j w[t][j] * Y[t][j],   Y[t][j] = expert_out[s_j] + (tokens[t] - centroids[s_j]),
// which is linear in the weights and in the restored rows:
//     grad_w[t][j]    = < grad_out[t], Y[t][j] >      (binary32)
//     grad_rows[t][j] = w[t][j] * grad_out[t]         (storage type, rounded once)
// One lane group per token.  The restored rows are formed as in the forward kernel and never stored; the k
// experts of a token are taken kBatch at a time so that their partial dot products stay in registers while the
// token's pieces are walked once per batch.  Each lane adds its pieces in ascending order, then the lanes of the
// group are added in a butterfly: the result does not depend on the launch.
constexpr int kBatch = 4;

template <typename DT, int LPR>
__global__ __launch_bounds__(256) void combine_backward_kernel(
    const char* __restrict__ tokens, const char* __restrict__ centroids, const char* __restrict__ expert_out,
    const int32_t* __restrict__ seg_of, const int32_t* __restrict__ seg_offsets, const float* __restrict__ gate_weight,
    const char* __restrict__ grad_out, float* __restrict__ grad_w, char* __restrict__ grad_rows, uint32_t T, uint32_t k,
    uint32_t cpr, uint32_t flags) {
  constexpr int G = 64 / LPR;
  constexpr int E = Piece<DT>::kElems;
  const uint32_t lane = threadIdx.x & 63;
  const uint64_t wave64 = linear_block() * 4u + (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (wave64 * G >= T) return;
  const uint32_t t = (uint32_t)(wave64 * G) + lane / LPR;   // below T + 64: 32 bits are enough
  const bool live = t < T;                                  // lanes of a dead group still take part in the butterfly
  const size_t row_bytes = (size_t)cpr * 16;
  const bool no_res = (flags & 1u) != 0;
  for (uint32_t j0 = 0; j0 < k; j0 += kBatch) {
    int32_t s[kBatch];
    float w[kBatch], dot[kBatch];
    bool on[kBatch], full[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      on[q] = live && j0 + q < k;
      const uint32_t a = on[q] ? t * k + j0 + q : 0u;
      s[q] = on[q] ? uniform<LPR>(seg_of[a]) : 0;
      w[q] = on[q] ? __int_as_float(uniform<LPR>(__float_as_int(gate_weight[a]))) : 0.0f;
      full[q] = on[q] && !no_res;
      if (full[q] && seg_offsets != nullptr)
        full[q] = uniform<LPR>(seg_offsets[s[q] + 1]) - uniform<LPR>(seg_offsets[s[q]]) != 1;
      dot[q] = 0.0f;
    }
    const bool any_full = full[0] || full[1] || full[2] || full[3];
    for (uint32_t c = lane % LPR; c < cpr && live; c += LPR) {
      float g[E], xv[E];
      Piece<DT>::widen(load16(grad_out + (size_t)t * row_bytes + c * 16), g);
      if (any_full) Piece<DT>::widen(load16(tokens + (size_t)t * row_bytes + c * 16), xv);
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        if (!on[q]) continue;
        float y[E];
        Piece<DT>::widen(load16(expert_out + (size_t)s[q] * row_bytes + c * 16), y);
        if (full[q]) {
          float cv[E];
          Piece<DT>::widen(load16(centroids + (size_t)s[q] * row_bytes + c * 16), cv);
#pragma unroll
          for (int i = 0; i < E; ++i) y[i] += xv[i] - cv[i];
        }
        float wg[E];
#pragma unroll
        for (int i = 0; i < E; ++i) {
          dot[q] = fmaf(g[i], y[i], dot[q]);
          wg[i] = w[q] * g[i];
        }
        store16_stream(grad_rows + ((size_t)t * k + j0 + q) * row_bytes + c * 16, Piece<DT>::narrow(wg));
      }
    }
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      float v = dot[q];
#pragma unroll
      for (int m = LPR / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
      if (on[q] && lane % LPR == 0) grad_w[(size_t)t * k + j0 + q] = v;
    }
  }
}

template <typename DT, int LPR>
void launch_combine_backward_lpr(const void* tokens, const void* centroids, const void* expert_out, const int32_t* seg_of,
                                 const int32_t* seg_offsets, const float* gate_weight, const void* grad_out, float* grad_w,
                                 void* grad_rows, int64_t T, int k, uint32_t cpr, uint32_t flags, hipStream_t stream) {
  constexpr int G = 64 / LPR;
  const uint64_t waves = ((uint64_t)T + G - 1) / G;
  const uint32_t blocks = (uint32_t)((waves + 3) / 4);
  hipLaunchKernelGGL((combine_backward_kernel<DT, LPR>), grid_of_blocks(blocks), dim3(256), 0, stream,
                     (const char*)tokens, (const char*)centroids, (const char*)expert_out, seg_of, seg_offsets, gate_weight,
                     (const char*)grad_out, grad_w, (char*)grad_rows, (uint32_t)T, (uint32_t)k, cpr, flags);
}

template <typename DT>
void launch_combine_backward_typed(const void* tokens, const void* centroids, const void* expert_out,
                                   const int32_t* seg_of, const int32_t* seg_offsets, const float* gate_weight,
                                   const void* grad_out, float* grad_w, void* grad_rows, int64_t T, int k, uint32_t cpr,
                                   uint32_t flags, hipStream_t stream) {
  if (cpr > 16)
    launch_combine_backward_lpr<DT, 64>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, grad_out, grad_w,
                                        grad_rows, T, k, cpr, flags, stream);
  else if (cpr > 4)
    launch_combine_backward_lpr<DT, 16>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, grad_out, grad_w,
                                        grad_rows, T, k, cpr, flags, stream);
  else
    launch_combine_backward_lpr<DT, 4>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, grad_out, grad_w,
                                       grad_rows, T, k, cpr, flags, stream);
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

hipError_t launch_combine_backward(const void* tokens, const void* centroids, const void* expert_out,
                                   const int32_t* seg_of, const int32_t* seg_offsets, const float* gate_weight,
                                   const void* grad_out, float* grad_w, void* grad_rows, int64_t T, int k, int d, bool bf16,
                                   uint32_t flags, hipStream_t stream) {
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  if (bf16)
    launch_combine_backward_typed<BF16>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, grad_out, grad_w,
                                        grad_rows, T, k, cpr, flags, stream);
  else
    launch_combine_backward_typed<F32>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, grad_out, grad_w,
                                       grad_rows, T, k, cpr, flags, stream);
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
