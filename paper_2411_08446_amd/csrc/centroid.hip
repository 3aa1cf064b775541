// Cluster centroids (Section 2.3 centroid formula with 1/n_j; Alg. 1 "Mean"):
// c_s = (1/n_s) * sum of the member rows, members taken in perm order,
// binary32 accumulation, one rounding to the storage type.
//
// HBM-bound gather: reads N token rows (T of them distinct), writes S rows.
// A group of LPR lanes owns one cluster and strides over the 16-byte pieces of
// the row; with rows of 1 KB and more that is a whole wave per cluster, and
// the cluster's offsets and member ids are wave-uniform scalars.  A one-member
// cluster is a plain row copy.  Centroid rows are written with streaming
// stores: nothing in this kernel reads them again.  By size: up to 16 members a
// plain sum, up to 32 a compensated one, up to kWindowMin the four waves of
// the workgroup share the cluster through LDS, beyond that the cluster is cut
// into blocks of positions that many workgroups (or waves) sum side by side;
// the one that finishes last adds the block sums in position order.
#include "kernels.h"

namespace lshmoe {

namespace {

constexpr int kPlainSumMax = 16;  // members summed without compensation
constexpr int kCoopMin = 32;      // clusters with more members (up to kWindowMin) are shared by the workgroup's waves
constexpr int kWindowMin = 1024;  // clusters with more members are cut into windows of kCentroidWindow positions
static_assert(kWindowMin >= kCentroidWindow, "a window meets at most two windowed clusters only if they are longer than it");
constexpr size_t kCoopMaxLds = 32 * 1024;  // more LDS per workgroup would cut the occupancy of the common path

template <int LPR> __device__ __forceinline__ int32_t uniform(int32_t v) {
  return LPR == 64 ? __builtin_amdgcn_readfirstlane(v) : v;  // a whole wave shares the value: keep it scalar
}

// Compensated sum of the token rows at sorted positions [a, b), wave-wide: lanes stride over the 16-byte pieces
// of the row, eight rows in flight (a walk by one wave is bound by memory latency).  emit(c, acc) receives the
// sums of piece c.  Kept small in registers on purpose: the kernel's occupancy is set by its largest path.
template <typename DT, typename Emit>
__device__ __forceinline__ void row_sum_kahan(const char* __restrict__ tokens, const int32_t* __restrict__ perm,
                                              int32_t a, int32_t b, uint32_t k, uint32_t cpr, size_t row_bytes,
                                              Emit emit) {
  constexpr int E = Piece<DT>::kElems;
  constexpr int kRows = 8;
  const uint32_t lane = threadIdx.x & 63;
  // every lane of the wave walks every pass, also lanes past the end of the row (they hold member ids, see
  // below, and only skip the row loads): the loop bounds are wave-uniform
  for (uint32_t c0 = 0; c0 < cpr; c0 += 64) {
    const uint32_t c = c0 + lane;
    const bool on = c < cpr;
    float acc[E], comp[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = comp[i] = 0.0f;
    // the member ids come 64 at a time, one coalesced load per block (lane l holds the id of row p0 + l), so
    // that a round of row loads does not wait for an id load first; the next block is fetched a block ahead
    int32_t ids = perm[min(a + (int32_t)lane, b - 1)];
    for (int32_t p0 = a; p0 < b; p0 += 64) {
      const int32_t ids_now = ids;
      if (p0 + 64 < b) ids = perm[min(p0 + 64 + (int32_t)lane, b - 1)];
      const int32_t rows_here = min(64, b - p0);
      for (int32_t j = 0; j < rows_here; j += kRows) {
        uint4 q[kRows];
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          const int32_t jj = min(j + u, rows_here - 1);  // the surplus rows of the last round are loaded and not added
          const uint32_t id = (uint32_t)__builtin_amdgcn_readlane(ids_now, jj);
          q[u] = on ? load16(tokens + (size_t)(id / k) * row_bytes + c * 16) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          if (j + u < rows_here) {
            float x[E];
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
    }
    if (on) emit(c, acc);
  }
}

// ... written as binary32 to out_row: the sum of one window of a long cluster.
template <typename DT>
__device__ __forceinline__ void window_sum(const char* __restrict__ tokens, const int32_t* __restrict__ perm,
                                           int32_t a, int32_t b, uint32_t k, uint32_t cpr, size_t row_bytes,
                                           float* __restrict__ out_row) {
  constexpr int E = Piece<DT>::kElems;
  row_sum_kahan<DT>(tokens, perm, a, b, k, cpr, row_bytes, [&](uint32_t c, const float (&acc)[E]) {
#pragma unroll
    for (int i = 0; i < E; i += 4)
      *(float4*)(out_row + (size_t)c * E + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
  });
}

// A cluster with more than kWindowMin members is summed by many waves: the sorted positions are cut into
// aligned blocks of kCentroidWindow; the wave that owns block m sums the part of the block that belongs to the
// long cluster containing the block's first position (slot 2m) and the part that belongs to a long cluster
// starting inside the block (slot 2m + 1; there is at most one, since a long cluster is longer than a block).
// Every window bumps its cluster's counter; the wave that brings it to the cluster's window count adds the
// partial sums in position order, so the result does not depend on which wave came last.
template <typename DT>
__device__ __forceinline__ void long_cluster_window(
    const char* __restrict__ tokens, const int32_t* __restrict__ perm, const int32_t* __restrict__ seg_offsets,
    char* __restrict__ centroids, float* partial, uint32_t* counters, int32_t s, int32_t a, int32_t b, uint32_t slot,
    uint32_t k, uint32_t cpr, uint32_t d, uint32_t mean) {
  constexpr int E = Piece<DT>::kElems;
  const size_t row_bytes = (size_t)cpr * 16;
  const uint32_t lane = threadIdx.x & 63;
  const int32_t lo = __builtin_amdgcn_readfirstlane(seg_offsets[s]);
  const int32_t hi = __builtin_amdgcn_readfirstlane(seg_offsets[s + 1]);
  window_sum<DT>(tokens, perm, a, b, k, cpr, row_bytes, partial + (size_t)slot * d);
  const uint32_t m0 = (uint32_t)lo / kCentroidWindow, m1 = (uint32_t)(hi - 1) / kCentroidWindow;
  const uint32_t first_slot = 2 * m0 + ((uint32_t)lo % kCentroidWindow != 0 ? 1u : 0u);
  __threadfence();  // the partial row is visible device-wide before the counter moves
  uint32_t old = 0;
  if (lane == 0) old = atomicAdd(&counters[first_slot], 1u);
  old = __builtin_amdgcn_readfirstlane(old);
  if (old != m1 - m0) return;
  __threadfence();  // last window of the cluster: every other partial row is complete and visible
  const uint32_t nwin = m1 - m0 + 1;
  const float fn = (float)(hi - lo);
  char* dst = centroids + (size_t)s * row_bytes;
  constexpr int kRows = 4;
  for (uint32_t c = lane; c < cpr; c += 64) {
    float acc[E], comp[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = comp[i] = 0.0f;
    for (uint32_t j = 0; j < nwin; j += kRows) {
      float x[kRows][E];
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        const uint32_t jj = min(j + u, nwin - 1);
        const float* src = partial + (size_t)(jj == 0 ? first_slot : 2 * (m0 + jj)) * d + (size_t)c * E;
#pragma unroll
        for (int i = 0; i < E; i += 4) {
          const float4 v = *(const float4*)(src + i);
          x[u][i] = v.x; x[u][i + 1] = v.y; x[u][i + 2] = v.z; x[u][i + 3] = v.w;
        }
      }
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        if (j + u < nwin) {
#pragma unroll
          for (int i = 0; i < E; ++i) {
            const float y = x[u][i] - comp[i];
            const float t = acc[i] + y;
            comp[i] = (t - acc[i]) - y;
            acc[i] = t;
          }
        }
      }
    }
    if (mean) {
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] /= fn;
    }
    store16_stream(dst + c * 16, Piece<DT>::narrow(acc));
  }
}


// The same with the four waves of a workgroup on one block of kWgWindow positions (needs the LDS of the shared
// sums): every wave sums its quarter of the block's part of the cluster into LDS, wave 0 adds the four in wave
// order, writes ONE partial row and bumps the counter - a quarter of the device-scope fences.  The workgroup that
// brings the counter to the cluster's block count adds the partial rows in position order, again a quarter per
// wave joined through LDS in wave order, so the result does not depend on which workgroup came last.
// Called by all four waves of the workgroup with the same arguments (barriers inside).
constexpr uint32_t kWgWindow = 2 * kCentroidWindow;   // measured: 128 and 512 positions per block are both slower
static_assert(kWgWindow <= (uint32_t)kWindowMin, "a block meets at most two clusters that are cut into blocks");

template <typename DT>
__device__ __forceinline__ void long_cluster_wg_window(
    const char* __restrict__ tokens, const int32_t* __restrict__ perm, const int32_t* __restrict__ seg_offsets,
    char* __restrict__ centroids, float* partial, uint32_t* counters, float* coop_sum, int32_t s, uint32_t block_p0,
    int32_t a, int32_t b, uint32_t slot, uint32_t k, uint32_t cpr, uint32_t d, uint32_t mean) {
  constexpr int E = Piece<DT>::kElems;
  const size_t row_bytes = (size_t)cpr * 16;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t w4 = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t* last_flag = reinterpret_cast<uint32_t*>(coop_sum + (size_t)4 * d);   // one word behind the four rows
  const int32_t qa = max(a, (int32_t)(block_p0 + w4 * (kWgWindow / 4)));
  const int32_t qb = min(b, (int32_t)(block_p0 + (w4 + 1) * (kWgWindow / 4)));
  float* mine = coop_sum + (size_t)w4 * d;
  if (qa < qb) {
    row_sum_kahan<DT>(tokens, perm, qa, qb, k, cpr, row_bytes, [&](uint32_t c, const float (&acc)[E]) {
#pragma unroll
      for (int i = 0; i < E; i += 4)
        *(float4*)(mine + (size_t)c * E + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
    });
  } else {
    for (uint32_t i = lane; i < d; i += 64) mine[i] = 0.0f;
  }
  const int32_t lo = __builtin_amdgcn_readfirstlane(seg_offsets[s]);
  const int32_t hi = __builtin_amdgcn_readfirstlane(seg_offsets[s + 1]);
  const uint32_t m0 = (uint32_t)lo / kWgWindow, m1 = (uint32_t)(hi - 1) / kWgWindow;
  const uint32_t first_slot = 2 * m0 + ((uint32_t)lo % kWgWindow != 0 ? 1u : 0u);
  __syncthreads();
  if (w4 == 0) {
    float* out_row = partial + (size_t)slot * d;
    for (uint32_t i = lane * 4; i < d; i += 256) {   // d is a multiple of 4
      float4 v = *(const float4*)(coop_sum + i);
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float4 u = *(const float4*)(coop_sum + (size_t)w * d + i);
        v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
      }
      *(float4*)(out_row + i) = v;
    }
    __threadfence();  // the partial row is visible device-wide before the counter moves
    if (lane == 0) *last_flag = atomicAdd(&counters[first_slot], 1u) == m1 - m0 ? 1u : 0u;
  }
  __syncthreads();    // the flag is set; the four LDS rows are free again
  if (*last_flag == 0u) return;   // the same for all four waves
  __threadfence();    // last block of the cluster: every other partial row is complete and visible
  const uint32_t nwin = m1 - m0 + 1;
  const uint32_t per = (nwin + 3) / 4;
  const uint32_t j0 = min(w4 * per, nwin), j1 = min(j0 + per, nwin);
  constexpr int kRows = 4;
  for (uint32_t c = lane; c < cpr; c += 64) {
    float acc[E], comp[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = comp[i] = 0.0f;
    for (uint32_t j = j0; j < j1; j += kRows) {
      float x[kRows][E];
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        const uint32_t jj = min(j + u, j1 - 1);
        const float* src = partial + (size_t)(jj == 0 ? first_slot : 2 * (m0 + jj)) * d + (size_t)c * E;
#pragma unroll
        for (int i = 0; i < E; i += 4) {
          const float4 v = *(const float4*)(src + i);
          x[u][i] = v.x; x[u][i + 1] = v.y; x[u][i + 2] = v.z; x[u][i + 3] = v.w;
        }
      }
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        if (j + u < j1) {
#pragma unroll
          for (int i = 0; i < E; ++i) {
            const float y = x[u][i] - comp[i];
            const float t = acc[i] + y;
            comp[i] = (t - acc[i]) - y;
            acc[i] = t;
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < E; i += 4)
      *(float4*)(mine + (size_t)c * E + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
  }
  __syncthreads();
  const float fn = (float)(hi - lo);
  char* dst = centroids + (size_t)s * row_bytes;
  for (uint32_t c = threadIdx.x; c < cpr; c += 256) {
    float acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) {
      acc[i] = coop_sum[(size_t)c * E + i];
#pragma unroll
      for (int w = 1; w < 4; ++w) acc[i] += coop_sum[((size_t)w * cpr + c) * E + i];
      if (mean) acc[i] /= fn;
    }
    store16_stream(dst + c * 16, Piece<DT>::narrow(acc));
  }
  __syncthreads();  // before the LDS rows are used again
}

template <typename DT, int LPR>
__global__ __launch_bounds__(256) void centroid_kernel(
    const char* __restrict__ tokens, const int32_t* __restrict__ perm, const int32_t* __restrict__ seg_offsets,
    const int32_t* __restrict__ seg_of, const int32_t* __restrict__ num_segments, char* __restrict__ centroids,
    float* partial, uint32_t* counters, uint32_t N, uint32_t k, uint32_t cpr, uint32_t mean, uint32_t coop) {
  constexpr int G = 64 / LPR;  // clusters handled side by side by one wave
  constexpr int E = Piece<DT>::kElems;
  extern __shared__ float coop_sum[];  // coop: [4 waves][cpr * E] partial sums of a cluster the workgroup shares
  const uint32_t S = (uint32_t)*num_segments;
  const uint32_t lane = threadIdx.x & 63;
  const uint64_t block64 = linear_block();
  if (block64 * 4u > (uint64_t)N) return;   // surplus workgroups of a folded grid (whole workgroup: no barrier is skipped by part of one)
  const uint32_t block = (uint32_t)block64;
  const uint32_t wave = block * 4u + (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t s = wave * G + lane / LPR;
  const size_t row_bytes = (size_t)cpr * 16;
  // Clusters of kCoopMin+1 .. kWindowMin members (whole-wave rows only): a single wave walking such a
  // cluster is bound by memory latency (one round of 8 rows per ~2 us), and when a few hundred of them hold
  // most of the assignments the kernel waits for them.  The four waves of the workgroup therefore share each
  // such cluster among the workgroup's four: a quarter of the members each, joined through LDS in wave order.
  const bool shares = LPR == 64 && coop != 0;
  auto shared_size = [&](int32_t n) { return shares && n > kCoopMin && n <= kWindowMin; };
  // the offsets of the workgroup's four clusters, fetched now (lane j holds the start of cluster 4*block + j,
  // clamped to the end) so that the sharing pass below does not start with a memory round trip
  // (read into scalars at once: waiting for this load later, behind the row stores, would keep the wave alive
  // until its stores have landed)
  int32_t wg_off[5] = {0, 0, 0, 0, 0};
  if (shares) {
    const int32_t v = seg_offsets[min(block * 4u + min(lane, 4u), S)];
#pragma unroll
    for (int j = 0; j < 5; ++j) wg_off[j] = __builtin_amdgcn_readlane(v, j);
  }
  // the sharing pass comes first: after its own cluster's stores a wave should have nothing left to wait for
  if (shares) {
    const uint32_t s0 = block * 4u, w4 = threadIdx.x >> 6;
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
      const uint32_t sj = s0 + j;
      if (sj >= S) break;  // the same for every wave of the workgroup
      const int32_t lo = wg_off[j], hi = wg_off[j + 1];
      const int32_t n = hi - lo;
      if (!shared_size(n)) continue;
      const int32_t quarter = (n + 3) / 4;
      const int32_t a = min(lo + (int32_t)w4 * quarter, hi), b = min(a + quarter, hi);
      float* mine = coop_sum + (size_t)w4 * cpr * E;
      if (a < b) {
        row_sum_kahan<DT>(tokens, perm, a, b, k, cpr, row_bytes, [&](uint32_t c, const float (&acc)[E]) {
#pragma unroll
          for (int i = 0; i < E; i += 4)
            *(float4*)(mine + (size_t)c * E + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
        });
      } else {
        for (uint32_t i = lane; i < cpr * E; i += 64) mine[i] = 0.0f;
      }
      __syncthreads();
      char* dst = centroids + (size_t)sj * row_bytes;
      const float fn = (float)n;
      for (uint32_t c = threadIdx.x; c < cpr; c += 256) {
        float acc[E];
#pragma unroll
        for (int i = 0; i < E; ++i) {
          acc[i] = coop_sum[(size_t)c * E + i];
#pragma unroll
          for (int w = 1; w < 4; ++w) acc[i] += coop_sum[((size_t)w * cpr + c) * E + i];
          if (mean) acc[i] /= fn;
        }
        store16_stream(dst + c * 16, Piece<DT>::narrow(acc));
      }
      __syncthreads();  // before the partial sums are overwritten
    }
  }
  if (s < S) {
    const int32_t lo = uniform<LPR>(seg_offsets[s]), hi = uniform<LPR>(seg_offsets[s + 1]);
    const int32_t n = hi - lo;
    if (shared_size(n)) {
      // left to the workgroup, below
    } else if (LPR == 64 && n > kPlainSumMax && n <= kWindowMin) {
      // a whole wave on a cluster of more than 16 members: compensated sum, eight rows in flight
      char* dst = centroids + (size_t)s * row_bytes;
      const float fn = (float)n;
      row_sum_kahan<DT>(tokens, perm, lo, hi, k, cpr, row_bytes, [&](uint32_t c, float (&acc)[E]) {
        if (mean) {
#pragma unroll
          for (int i = 0; i < E; ++i) acc[i] /= fn;
        }
        store16_stream(dst + c * 16, Piece<DT>::narrow(acc));
      });
    } else if (n <= kWindowMin) {
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
          // longer cluster: compensated (Kahan) summation keeps the binary32 sum within
          // a couple of ulps of the exact one however many members there are
          float comp[E];
#pragma unroll
          for (int i = 0; i < E; ++i) comp[i] = 0.0f;
          for (; p < hi; p += 4) {
            uint4 q[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
              if (p + u < hi)
                q[u] = load16(tokens + (size_t)((uint32_t)uniform<LPR>(perm[p + u]) / k) * row_bytes + c * 16);
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
        if (mean) {
          const float fn = (float)n;
#pragma unroll
          for (int i = 0; i < E; ++i) acc[i] /= fn;
        }
        store16_stream(dst + c * 16, Piece<DT>::narrow(acc));
      }
    }
  }
  if (shares) {
    // window duty with the workgroup's LDS rows: workgroup m looks after block m of 4 * kCentroidWindow positions
    // (every wave of the workgroup gets here: nothing above returns for a single wave)
    if ((uint64_t)block * kWgWindow >= N) return;
    const uint32_t p0 = block * kWgWindow, p1 = min(p0 + kWgWindow, N);
    const uint32_t d = cpr * E;
    const int32_t sf = __builtin_amdgcn_readfirstlane(seg_of[perm[p0]]);
    const int32_t sl = __builtin_amdgcn_readfirstlane(seg_of[perm[p1 - 1]]);
    {
      const int32_t lo = __builtin_amdgcn_readfirstlane(seg_offsets[sf]);
      const int32_t hi = __builtin_amdgcn_readfirstlane(seg_offsets[sf + 1]);
      if (hi - lo > kWindowMin)
        long_cluster_wg_window<DT>(tokens, perm, seg_offsets, centroids, partial, counters, coop_sum, sf, p0, (int32_t)p0,
                                   min(hi, (int32_t)p1), 2 * block, k, cpr, d, mean);
    }
    if (sl != sf) {
      const int32_t lo = __builtin_amdgcn_readfirstlane(seg_offsets[sl]);
      const int32_t hi = __builtin_amdgcn_readfirstlane(seg_offsets[sl + 1]);
      if (hi - lo > kWindowMin)
        long_cluster_wg_window<DT>(tokens, perm, seg_offsets, centroids, partial, counters, coop_sum, sl, p0, lo,
                                   (int32_t)p1, 2 * block + 1, k, cpr, d, mean);
    }
    return;
  }
  // window duty: wave m looks after block m of the sorted positions
  if ((uint64_t)wave * kCentroidWindow >= N) return;
  const uint32_t p0 = wave * (uint32_t)kCentroidWindow;
  const uint32_t p1 = min(p0 + (uint32_t)kCentroidWindow, N);
  const uint32_t d = cpr * E;
  const int32_t sf = __builtin_amdgcn_readfirstlane(seg_of[perm[p0]]);
  const int32_t sl = __builtin_amdgcn_readfirstlane(seg_of[perm[p1 - 1]]);
  {
    const int32_t lo = __builtin_amdgcn_readfirstlane(seg_offsets[sf]);
    const int32_t hi = __builtin_amdgcn_readfirstlane(seg_offsets[sf + 1]);
    if (hi - lo > kWindowMin)
      long_cluster_window<DT>(tokens, perm, seg_offsets, centroids, partial, counters, sf, (int32_t)p0,
                              min(hi, (int32_t)p1), 2 * wave, k, cpr, d, mean);
  }
  if (sl != sf) {
    const int32_t lo = __builtin_amdgcn_readfirstlane(seg_offsets[sl]);
    const int32_t hi = __builtin_amdgcn_readfirstlane(seg_offsets[sl + 1]);
    if (hi - lo > kWindowMin)
      long_cluster_window<DT>(tokens, perm, seg_offsets, centroids, partial, counters, sl, lo, (int32_t)p1,
                              2 * wave + 1, k, cpr, d, mean);
  }
}

template <typename DT, int LPR>
void launch_lpr(const void* tokens, const int32_t* perm, const int32_t* seg_offsets, const int32_t* seg_of,
                const int32_t* num_segments, void* centroids, float* partial, uint32_t* counters, int64_t N, int k,
                uint32_t cpr, bool mean, hipStream_t stream) {
  constexpr int G = 64 / LPR;
  const uint64_t waves = ((uint64_t)N + G - 1) / G;  // worst case S == N; surplus waves leave at once
  const uint32_t blocks = (uint32_t)((waves + 3) / 4);
  const size_t coop_bytes = (size_t)4 * cpr * Piece<DT>::kElems * sizeof(float);  // four partial rows in binary32
  const bool coop = LPR == 64 && coop_bytes <= kCoopMaxLds;
  hipLaunchKernelGGL((centroid_kernel<DT, LPR>), grid_of_blocks(blocks), dim3(256), coop ? coop_bytes + 16 : 0, stream,
                     (const char*)tokens, perm, seg_offsets, seg_of, num_segments, (char*)centroids, partial, counters,
                     (uint32_t)N, (uint32_t)k, cpr, mean ? 1u : 0u, coop ? 1u : 0u);
}

template <typename DT>
void launch_typed(const void* tokens, const int32_t* perm, const int32_t* seg_offsets, const int32_t* seg_of,
                  const int32_t* num_segments, void* centroids, float* partial, uint32_t* counters, int64_t N, int k,
                  uint32_t cpr, bool mean, hipStream_t stream) {
  if (cpr > 16)
    launch_lpr<DT, 64>(tokens, perm, seg_offsets, seg_of, num_segments, centroids, partial, counters, N, k, cpr, mean, stream);
  else if (cpr > 4)
    launch_lpr<DT, 16>(tokens, perm, seg_offsets, seg_of, num_segments, centroids, partial, counters, N, k, cpr, mean, stream);
  else
    launch_lpr<DT, 4>(tokens, perm, seg_offsets, seg_of, num_segments, centroids, partial, counters, N, k, cpr, mean, stream);
}

}  // namespace

hipError_t launch_centroid(const void* tokens, const int32_t* perm, const int32_t* seg_offsets, const int32_t* seg_of,
                           const int32_t* num_segments, void* centroids, float* partial, uint32_t* counters, int64_t N,
                           int k, int d, bool bf16, bool mean, hipStream_t stream) {
  const uint32_t cpr = (uint32_t)((size_t)d * (bf16 ? 2 : 4) / 16);
  if (bf16)
    launch_typed<BF16>(tokens, perm, seg_offsets, seg_of, num_segments, centroids, partial, counters, N, k, cpr, mean, stream);
  else
    launch_typed<F32>(tokens, perm, seg_offsets, seg_of, num_segments, centroids, partial, counters, N, k, cpr, mean, stream);
  return hipGetLastError();
}

}  // namespace lshmoe
