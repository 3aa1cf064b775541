// Restore with residual compensation (Eq. 4 and Eq. 5):
//     out[a] = expert_out[s] + (tokens[a / k] - centroids[s]),   s = seg_of[a].
//
// HBM-bound gather: per output row it reads the expert-output row and, for
// members of clusters with more than one member, the token row and the
// centroid row; it writes one row.  A group of LPR lanes owns kRows
// consecutive output rows (the k assignments of a token are consecutive, so
// they share the token row) and strides over the 16-byte pieces; with rows of
// 1 KB and more that is a whole wave, and the cluster lookups are wave-uniform
// scalars.  Output rows are written with streaming stores.
#include "kernels.h"

namespace lshmoe {

namespace {

constexpr int kRows = 2;  // output rows a lane group works on at once

template <int LPR> __device__ __forceinline__ int32_t uniform(int32_t v) {
  return LPR == 64 ? __builtin_amdgcn_readfirstlane(v) : v;
}

// With perm and num_segments given, the lane groups walk the rows in cluster order (row a = perm[p]) when the
// clusters are long on average (S / N below kClusterOrderBelow): the members of a cluster are then restored
// side by side and its expert-output and centroid rows are fetched from memory once instead of once per
// member.  With mostly one-member clusters the assignment order is faster (measured at T5: S/N 0.92:
// 101 against 106 us; S/N 0.38: 124 against 104 us).
constexpr uint32_t kClusterOrderBelowNum = 13, kClusterOrderBelowDen = 20;  // S / N < 0.65

template <typename DT, int LPR>
__global__ __launch_bounds__(256) void restore_kernel(
    const char* __restrict__ tokens, const char* __restrict__ centroids, const char* __restrict__ expert_out,
    const int32_t* __restrict__ seg_of, const int32_t* __restrict__ seg_offsets, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ num_segments, char* __restrict__ out, uint32_t N, uint32_t k, uint32_t cpr,
    uint32_t flags) {
  constexpr int G = 64 / LPR;
  constexpr int E = Piece<DT>::kElems;
  const uint32_t lane = threadIdx.x & 63;
  // a folded grid can pass 2^32 threads: the workgroup's first row is checked in 64 bits, the rest fits 32.
  // The row index is left in a vector register on purpose: with a scalar index the cluster lookups below
  // become scalar-cache loads, and this kernel then runs 3 us slower at the T5 shape (the gate-weighted
  // variant and the token-gradient kernel, which have one more lookup per row, gain from the scalar form).
  const uint64_t block64 = linear_block();
  if (block64 * (4u * G * kRows) >= N) return;
  const uint32_t a0 = (((uint32_t)block64 * 4u + (threadIdx.x >> 6)) * G + lane / LPR) * kRows;
  if (a0 >= N) return;
  const size_t row_bytes = (size_t)cpr * 16;
  const bool no_res = (flags & 1u) != 0;

  bool by_cluster = false;
  if (perm != nullptr && num_segments != nullptr)
    by_cluster = (uint64_t)(uint32_t)*num_segments * kClusterOrderBelowDen < (uint64_t)N * kClusterOrderBelowNum;
  int32_t s[kRows];
  uint32_t a[kRows];   // the rows this lane group restores
  bool live[kRows], full[kRows];
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    live[u] = a0 + u < N;
    a[u] = a0 + u;
    if (by_cluster && live[u]) a[u] = (uint32_t)uniform<LPR>(perm[a0 + u]);
    s[u] = live[u] ? uniform<LPR>(seg_of[a[u]]) : 0;
  }
#pragma unroll
  for (int u = 0; u < kRows; ++u) {
    full[u] = live[u] && !no_res;
    // a one-member cluster's centroid is its token bit for bit: the residual is exactly zero
    if (full[u] && seg_offsets != nullptr)
      full[u] = uniform<LPR>(seg_offsets[s[u] + 1]) - uniform<LPR>(seg_offsets[s[u]]) != 1;
  }
  for (uint32_t c = lane % LPR; c < cpr; c += LPR) {
    uint4 ec[kRows], x[kRows], cc[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      if (live[u]) ec[u] = load16(expert_out + (size_t)s[u] * row_bytes + c * 16);
      if (full[u]) {
        x[u] = load16(tokens + (size_t)(a[u] / k) * row_bytes + c * 16);
        cc[u] = load16(centroids + (size_t)s[u] * row_bytes + c * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      if (!live[u]) continue;
      uint4 y = ec[u];
      if (!no_res) {
        float e[E], xv[E], cv[E];
        Piece<DT>::widen(ec[u], e);
        if (full[u]) {
          Piece<DT>::widen(x[u], xv);
          Piece<DT>::widen(cc[u], cv);
#pragma unroll
          for (int i = 0; i < E; ++i) e[i] += xv[i] - cv[i];
        } else {
#pragma unroll
          for (int i = 0; i < E; ++i) e[i] += 0.0f;  // e + (+0): only turns -0 into +0, as the full formula would
        }
        y = Piece<DT>::narrow(e);
      }
      store16_stream(out + (size_t)a[u] * row_bytes + c * 16, y);
    }
  }
}

// Restore fused with the gate-weighted combine of the k expert outputs of a token (Eq. 2 with gate weights):
//     out[t] = sum_j w[t][j] * (expert_out[s_j] + (tokens[t] - centroids[s_j])),   s_j = seg_of[t*k + j],
// accumulated in binary32 in the order j = 0..k-1 and rounded once.  One lane group per token: the token row
// is read once, and one row is written instead of k.
template <typename DT, int LPR>
__global__ __launch_bounds__(256) void restore_combine_kernel(
    const char* __restrict__ tokens, const char* __restrict__ centroids, const char* __restrict__ expert_out,
    const int32_t* __restrict__ seg_of, const int32_t* __restrict__ seg_offsets, const float* __restrict__ gate_weight,
    char* __restrict__ out, uint32_t T, uint32_t k, uint32_t cpr, uint32_t flags) {
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
    float acc[E], xv[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.0f;
    bool have_x = false;
    for (uint32_t j = 0; j < k; ++j) {
      const int32_t s = uniform<LPR>(seg_of[t * k + j]);
      const float w = __int_as_float(uniform<LPR>(__float_as_int(gate_weight[t * k + j])));
      bool full = !no_res;
      if (full && seg_offsets != nullptr)
        full = uniform<LPR>(seg_offsets[s + 1]) - uniform<LPR>(seg_offsets[s]) != 1;
      float e[E];
      Piece<DT>::widen(load16(expert_out + (size_t)s * row_bytes + c * 16), e);
      if (full) {
        if (!have_x) {
          Piece<DT>::widen(load16(tokens + (size_t)t * row_bytes + c * 16), xv);
          have_x = true;
        }
        float cv[E];
        Piece<DT>::widen(load16(centroids + (size_t)s * row_bytes + c * 16), cv);
#pragma unroll
        for (int i = 0; i < E; ++i) e[i] += xv[i] - cv[i];
      }
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] = fmaf(w, e[i], acc[i]);
    }
    store16_stream(out + (size_t)t * row_bytes + c * 16, Piece<DT>::narrow(acc));
  }
}

template <typename DT, int LPR>
void launch_combine_lpr(const void* tokens, const void* centroids, const void* expert_out, const int32_t* seg_of,
                        const int32_t* seg_offsets, const float* gate_weight, void* out, int64_t T, int k,
                        uint32_t cpr, uint32_t flags, hipStream_t stream) {
  constexpr int G = 64 / LPR;
  const uint64_t waves = ((uint64_t)T + G - 1) / G;
  const uint32_t blocks = (uint32_t)((waves + 3) / 4);
  hipLaunchKernelGGL((restore_combine_kernel<DT, LPR>), grid_of_blocks(blocks), dim3(256), 0, stream, (const char*)tokens,
                     (const char*)centroids, (const char*)expert_out, seg_of, seg_offsets, gate_weight, (char*)out,
                     (uint32_t)T, (uint32_t)k, cpr, flags);
}

template <typename DT>
void launch_combine_typed(const void* tokens, const void* centroids, const void* expert_out, const int32_t* seg_of,
                          const int32_t* seg_offsets, const float* gate_weight, void* out, int64_t T, int k,
                          uint32_t cpr, uint32_t flags, hipStream_t stream) {
  if (cpr > 16)
    launch_combine_lpr<DT, 64>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, out, T, k, cpr, flags, stream);
  else if (cpr > 4)
    launch_combine_lpr<DT, 16>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, out, T, k, cpr, flags, stream);
  else
    launch_combine_lpr<DT, 4>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, out, T, k, cpr, flags, stream);
}

template <typename DT, int LPR>
void launch_lpr(const void* tokens, const void* centroids, const void* expert_out, const int32_t* seg_of,
                const int32_t* seg_offsets, const int32_t* perm, const int32_t* num_segments, void* out, int64_t N,
                int k, uint32_t cpr, uint32_t flags, hipStream_t stream) {
  constexpr int G = 64 / LPR;
  const uint64_t groups = ((uint64_t)N + kRows - 1) / kRows;
  const uint64_t waves = (groups + G - 1) / G;
  const uint32_t blocks = (uint32_t)((waves + 3) / 4);
  hipLaunchKernelGGL((restore_kernel<DT, LPR>), grid_of_blocks(blocks), dim3(256), 0, stream, (const char*)tokens,
                     (const char*)centroids, (const char*)expert_out, seg_of, seg_offsets, perm, num_segments,
                     (char*)out, (uint32_t)N, (uint32_t)k, cpr, flags);
}

template <typename DT>
void launch_typed(const void* tokens, const void* centroids, const void* expert_out, const int32_t* seg_of,
                  const int32_t* seg_offsets, const int32_t* perm, const int32_t* num_segments, void* out, int64_t N,
                  int k, uint32_t cpr, uint32_t flags, hipStream_t stream) {
  if (cpr > 16)
    launch_lpr<DT, 64>(tokens, centroids, expert_out, seg_of, seg_offsets, perm, num_segments, out, N, k, cpr, flags, stream);
  else if (cpr > 4)
    launch_lpr<DT, 16>(tokens, centroids, expert_out, seg_of, seg_offsets, perm, num_segments, out, N, k, cpr, flags, stream);
  else
    launch_lpr<DT, 4>(tokens, centroids, expert_out, seg_of, seg_offsets, perm, num_segments, out, N, k, cpr, flags, stream);
}

}  // namespace

hipError_t launch_restore(const void* tokens, const void* centroids, const void* expert_out,
                          const int32_t* seg_of, const int32_t* seg_offsets, const int32_t* perm,
                          const int32_t* num_segments, void* out, int64_t N, int k, int d, bool bf16, uint32_t flags,
                          hipStream_t stream) {
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  if (bf16)
    launch_typed<BF16>(tokens, centroids, expert_out, seg_of, seg_offsets, perm, num_segments, out, N, k, cpr, flags, stream);
  else
    launch_typed<F32>(tokens, centroids, expert_out, seg_of, seg_offsets, perm, num_segments, out, N, k, cpr, flags, stream);
  return hipGetLastError();
}

hipError_t launch_restore_combine(const void* tokens, const void* centroids, const void* expert_out,
                                  const int32_t* seg_of, const int32_t* seg_offsets, const float* gate_weight,
                                  void* out, int64_t T, int k, int d, bool bf16, uint32_t flags, hipStream_t stream) {
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  if (bf16)
    launch_combine_typed<BF16>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, out, T, k, cpr, flags, stream);
  else
    launch_combine_typed<F32>(tokens, centroids, expert_out, seg_of, seg_offsets, gate_weight, out, T, k, cpr, flags, stream);
  return hipGetLastError();
}

}  // namespace lshmoe
