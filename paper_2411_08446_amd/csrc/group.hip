// Grouping of assignments by (expert, bucket) (Alg. 1: dispatch, then split
// each expert's tokens into clusters by bucket id).
//
// A stable least-significant-digit radix sort of the packed key
// (expert << bbits | bucket) carrying the assignment index, 8 bits per pass,
// followed by a head-flag scan that numbers the clusters.  Integer work only;
// every result is deterministic.  The arrays are a few MB at most, so the
// step is bound by launch latency rather than by HBM.
//
// Per pass:  tile histogram -> exclusive scan of the (bin, tile) table ->
// scatter.  Ranks inside a tile come from wave ballots: a wave of 64 keys
// finds, for every lane, the lanes holding the same digit; tile order equals
// element order, which keeps the sort stable.
#include "kernels.h"

namespace lshmoe {

namespace {

constexpr int kBins = 256;
constexpr int kSortThreads = 256;
constexpr int kSortItems = kSortTile / kSortThreads;  // 8
constexpr int kGroupsPerTile = kSortTile / kWave;     // 32 waves' worth of keys
constexpr int kSegThreads = 256;
constexpr int kSegItems = kSegTile / kSegThreads;     // 4

struct KeySource {
  // pass 0 builds keys from the inputs; later passes read the ping-pong buffers
  const int32_t* expert;
  const uint64_t* bucket;
  const uint64_t* key;
  const int32_t* idx;
  uint32_t k, E;
  int bbits;
};

template <bool FIRST>
__device__ __forceinline__ void load_item(const KeySource& src, uint32_t i, uint64_t& key, int32_t& idx) {
  if (FIRST) {
    uint32_t e = (uint32_t)src.expert[i];
    if (e >= src.E) e = src.E - 1;  // out-of-range ids violate the contract; stay in bounds
    key = ((uint64_t)e << src.bbits) | src.bucket[i / src.k];
    idx = (int32_t)i;
  } else {
    key = src.key[i];
    idx = src.idx[i];
  }
}

template <bool FIRST>
__global__ __launch_bounds__(kSortThreads) void sort_hist_kernel(KeySource src, uint32_t N, int shift,
                                                                 uint32_t nblk, uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[kBins];
  h[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * kSortTile;
#pragma unroll
  for (int it = 0; it < kSortItems; ++it) {
    const uint32_t i = base + it * kSortThreads + threadIdx.x;
    if (i < N) {
      uint64_t key;
      int32_t idx;
      load_item<FIRST>(src, i, key, idx);
      atomicAdd(&h[(uint32_t)(key >> shift) & (kBins - 1)], 1u);
    }
  }
  __syncthreads();
  hist[threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];  // bin-major: a scan over the table orders by (bin, tile)
}

// In-place exclusive scan of n 32-bit counters by one workgroup of 1024
// threads: the array is walked in slabs of 4096 counters (one coalesced
// 16-byte load per thread), carrying the running total from slab to slab.
__global__ __launch_bounds__(1024) void scan_kernel(uint32_t* __restrict__ data, uint32_t n) {
  __shared__ uint32_t wave_sum[16];
  __shared__ uint32_t carry_s;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t carry = 0;
  for (uint32_t base = 0; base < n; base += 4096) {
    const uint32_t i = base + threadIdx.x * 4;
    uint32_t v[4] = {0, 0, 0, 0};
    if (i + 4 <= n) {
      const uint4 q = *reinterpret_cast<const uint4*>(data + i);
      v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    } else {
      for (int j = 0; j < 4; ++j)
        if (i + j < n) v[j] = data[i + j];
    }
    const uint32_t sum = v[0] + v[1] + v[2] + v[3];
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    uint32_t run = carry + inc - sum;
#pragma unroll
    for (int w = 0; w < 16; ++w)
      if (w < wave) run += wave_sum[w];
    if (threadIdx.x == 1023) carry_s = run + sum;
    uint32_t o[4];
    o[0] = run; o[1] = o[0] + v[0]; o[2] = o[1] + v[1]; o[3] = o[2] + v[2];
    if (i + 4 <= n) {
      *reinterpret_cast<uint4*>(data + i) = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
      for (int j = 0; j < 4; ++j)
        if (i + j < n) data[i + j] = o[j];
    }
    __syncthreads();
    carry = carry_s;
  }
}

template <bool FIRST>
__global__ __launch_bounds__(kSortThreads) void sort_scatter_kernel(KeySource src, uint32_t N, int shift,
                                                                    uint32_t nblk, const uint32_t* __restrict__ hist,
                                                                    uint64_t* __restrict__ dst_key,
                                                                    int32_t* __restrict__ dst_idx) {
  __shared__ uint32_t gh[kGroupsPerTile][kBins];  // per 64-key group digit counts, then start offsets
  for (int i = threadIdx.x; i < kGroupsPerTile * kBins; i += kSortThreads) (&gh[0][0])[i] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * kSortTile;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  uint64_t key[kSortItems];
  int32_t idx[kSortItems];
  uint32_t rank[kSortItems];
#pragma unroll
  for (int it = 0; it < kSortItems; ++it) {
    const uint32_t i = base + it * kSortThreads + threadIdx.x;
    const bool valid = i < N;
    key[it] = 0;
    idx[it] = 0;
    if (valid) load_item<FIRST>(src, i, key[it], idx[it]);
    const uint32_t digit = (uint32_t)(key[it] >> shift) & (kBins - 1);
    uint64_t same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (digit >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      same &= bit ? bal : ~bal;
    }
    rank[it] = (uint32_t)__popcll(same & lt_mask);
    if (valid && rank[it] == 0) gh[it * (kSortThreads / kWave) + wave][digit] = (uint32_t)__popcll(same);
  }
  __syncthreads();
  {
    const int bin = threadIdx.x;
    uint32_t run = hist[bin * nblk + blockIdx.x];
#pragma unroll 8
    for (int g = 0; g < kGroupsPerTile; ++g) {
      const uint32_t c = gh[g][bin];
      gh[g][bin] = run;
      run += c;
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kSortItems; ++it) {
    const uint32_t i = base + it * kSortThreads + threadIdx.x;
    if (i < N) {
      const uint32_t digit = (uint32_t)(key[it] >> shift) & (kBins - 1);
      const uint32_t pos = gh[it * (kSortThreads / kWave) + wave][digit] + rank[it];
      dst_key[pos] = key[it];
      dst_idx[pos] = idx[it];
    }
  }
}

// Exclusive scan of one value per thread across a 256-thread block.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sum /*[4]*/, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wave_sum[wave] = inc;
  __syncthreads();
  uint32_t before = 0;
  total = 0;
#pragma unroll
  for (int w = 0; w < kSegThreads / kWave; ++w) {
    if (w < wave) before += wave_sum[w];
    total += wave_sum[w];
  }
  __syncthreads();
  return before + inc - v;
}

__device__ __forceinline__ bool is_head(const uint64_t* __restrict__ key, uint32_t p) {
  return p == 0 || key[p] != key[p - 1];
}

__global__ __launch_bounds__(kSegThreads) void seg_count_kernel(const uint64_t* __restrict__ key, uint32_t N,
                                                                uint32_t nblk, uint32_t* __restrict__ blocksum) {
  __shared__ uint32_t wave_sum[kSegThreads / kWave];
  const uint32_t base = blockIdx.x * kSegTile + threadIdx.x * kSegItems;
  uint32_t c = 0;
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) {
    const uint32_t p = base + it;
    if (p < N && is_head(key, p)) ++c;
  }
  uint32_t total;
  block_exclusive_scan(c, wave_sum, total);
  if (threadIdx.x == 0) {
    blocksum[blockIdx.x] = total;
    if (blockIdx.x == 0) blocksum[nblk] = 0;  // after the scan this slot holds the grand total
  }
}

__global__ __launch_bounds__(kSegThreads) void seg_write_kernel(
    const uint64_t* __restrict__ key, const int32_t* __restrict__ perm, uint32_t N, uint32_t E, int bbits,
    const uint32_t* __restrict__ blocksum, int32_t* __restrict__ seg_offsets, int32_t* __restrict__ seg_expert,
    int32_t* __restrict__ expert_offsets, int32_t* __restrict__ seg_of, int32_t* __restrict__ num_segments) {
  __shared__ uint32_t wave_sum[kSegThreads / kWave];
  const uint32_t base = blockIdx.x * kSegTile + threadIdx.x * kSegItems;
  bool head[kSegItems];
  uint32_t c = 0;
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) {
    const uint32_t p = base + it;
    head[it] = p < N && is_head(key, p);
    c += head[it] ? 1u : 0u;
  }
  uint32_t total;
  uint32_t seg = blocksum[blockIdx.x] + block_exclusive_scan(c, wave_sum, total);  // heads before this thread
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) {
    const uint32_t p = base + it;
    if (p >= N) break;
    if (head[it]) {
      const uint32_t e = (uint32_t)(key[p] >> bbits);
      seg_offsets[seg] = (int32_t)p;
      seg_expert[seg] = (int32_t)e;
      const uint32_t first = p == 0 ? 0u : (uint32_t)(key[p - 1] >> bbits) + 1u;
      for (uint32_t x = first; x <= e; ++x) expert_offsets[x] = (int32_t)seg;  // experts that start (or are empty) here
      ++seg;
    }
    seg_of[perm[p]] = (int32_t)(seg - 1);
    if (p == N - 1) {
      const uint32_t e = (uint32_t)(key[p] >> bbits);
      for (uint32_t x = e + 1; x <= E; ++x) expert_offsets[x] = (int32_t)seg;
      seg_offsets[seg] = (int32_t)N;
      *num_segments = (int32_t)seg;
    }
  }
}

int bits_for(uint64_t max_value) {  // number of bits needed to hold max_value
  int b = 0;
  while (max_value) {
    ++b;
    max_value >>= 1;
  }
  return b;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

bool plan_group(int64_t T, int k, int E, int L, int r, GroupPlan* plan) {
  uint64_t nb = 1;  // (2r)^L, known to be < 2^63 by the caller's check
  for (int l = 0; l < L; ++l) nb *= (uint64_t)(2 * r);
  GroupPlan p{};
  p.N = T * k;
  p.ebits = bits_for((uint64_t)E - 1);
  p.bbits = bits_for(nb - 1);
  if (p.ebits + p.bbits > 64) return false;
  p.passes = (p.ebits + p.bbits + 7) / 8;
  if (p.passes < 1) p.passes = 1;
  p.sort_blocks = (uint32_t)((p.N + kSortTile - 1) / kSortTile);
  p.seg_blocks = (uint32_t)((p.N + kSegTile - 1) / kSegTile);
  size_t off = 0;
  for (int i = 0; i < 2; ++i) {
    p.off_key[i] = off;
    off = align256(off + (size_t)p.N * 8);
  }
  for (int i = 0; i < 2; ++i) {
    p.off_idx[i] = off;
    off = align256(off + (size_t)p.N * 4);
  }
  p.off_hist = off;
  off = align256(off + (size_t)kBins * p.sort_blocks * 4);
  p.off_blocksum = off;
  off = align256(off + ((size_t)p.seg_blocks + 1) * 4);
  p.total_bytes = off;
  *plan = p;
  return true;
}

hipError_t launch_group(const GroupPlan& plan, const int32_t* expert, const uint64_t* bucket, int k, int E,
                        int32_t* seg_offsets, int32_t* seg_expert, int32_t* expert_offsets, int32_t* perm,
                        int32_t* seg_of, int32_t* num_segments, char* ws, hipStream_t stream) {
  const uint32_t N = (uint32_t)plan.N;
  uint64_t* keybuf[2] = {(uint64_t*)(ws + plan.off_key[0]), (uint64_t*)(ws + plan.off_key[1])};
  int32_t* idxbuf[2] = {(int32_t*)(ws + plan.off_idx[0]), (int32_t*)(ws + plan.off_idx[1])};
  uint32_t* hist = (uint32_t*)(ws + plan.off_hist);
  uint32_t* blocksum = (uint32_t*)(ws + plan.off_blocksum);
  const uint32_t nblk = plan.sort_blocks;

  KeySource src{expert, bucket, nullptr, nullptr, (uint32_t)k, (uint32_t)E, plan.bbits};
  const uint64_t* sorted_key = nullptr;
  for (int p = 0; p < plan.passes; ++p) {
    const bool last = p == plan.passes - 1;
    uint64_t* dkey = keybuf[p & 1];
    int32_t* didx = last ? perm : idxbuf[p & 1];
    const int shift = 8 * p;
    if (p == 0) {
      hipLaunchKernelGGL(sort_hist_kernel<true>, dim3(nblk), dim3(kSortThreads), 0, stream, src, N, shift, nblk, hist);
      hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, stream, hist, (uint32_t)kBins * nblk);
      hipLaunchKernelGGL(sort_scatter_kernel<true>, dim3(nblk), dim3(kSortThreads), 0, stream, src, N, shift, nblk,
                         hist, dkey, didx);
    } else {
      hipLaunchKernelGGL(sort_hist_kernel<false>, dim3(nblk), dim3(kSortThreads), 0, stream, src, N, shift, nblk, hist);
      hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, stream, hist, (uint32_t)kBins * nblk);
      hipLaunchKernelGGL(sort_scatter_kernel<false>, dim3(nblk), dim3(kSortThreads), 0, stream, src, N, shift, nblk,
                         hist, dkey, didx);
    }
    src.key = dkey;
    src.idx = didx;
    sorted_key = dkey;
  }
  const uint32_t sblk = plan.seg_blocks;
  hipLaunchKernelGGL(seg_count_kernel, dim3(sblk), dim3(kSegThreads), 0, stream, sorted_key, N, sblk, blocksum);
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, stream, blocksum, sblk + 1);
  hipLaunchKernelGGL(seg_write_kernel, dim3(sblk), dim3(kSegThreads), 0, stream, sorted_key, perm, N, (uint32_t)E,
                     plan.bbits, blocksum, seg_offsets, seg_expert, expert_offsets, seg_of, num_segments);
  return hipGetLastError();
}

}  // namespace lshmoe
