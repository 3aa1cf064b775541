// Grouping of assignments by (expert, bucket) (Alg. 1: dispatch, then split
// each expert's tokens into clusters by bucket id).
//
// A stable sort of the packed key (expert << bbits | bucket) carrying the
// assignment index, followed by a head-flag pass that numbers the clusters.
// Integer work only; every result is deterministic.  The arrays are a few MB
// at most, so the step is bound by launch latency, not by HBM: the design goal
// is few kernels.  Three routes by size:
//
//  - up to kSmallMaxN assignments: everything in one workgroup and one launch.
//  - up to kFusedMaxTiles tiles of 2048 (every paper-shaped layer): ONE global
//    radix pass on the top 9 key bits (histogram kernel + scatter kernel; the
//    histogram kernel writes the tile's digit counts as one row of a tile-major
//    table and every scatter block derives its own output offsets from that
//    small table, so there is no scan launch), then one launch that sorts every
//    bin on the remaining bits inside LDS (in chunks of 2048 keys), one launch
//    that merges the chunks of bins that have several (it leaves at once when
//    there are none), and one launch that numbers the clusters from the head
//    counts the two bin kernels left per tile: five launches whatever the key
//    width.  (Before: a histogram and a scatter launch per 9 key bits, and a
//    counting launch.)
//  - larger: least-significant-digit radix passes of histogram,
//    single-workgroup scan of the (bin, tile) table and scatter.
//
// Ranks inside a tile of 2048 keys come from wave ballots: a wave of 64 keys
// finds, for every lane, the lanes holding the same digit; tile order equals
// element order, which keeps the sort stable.  (Accumulating the next pass's
// table with global atomics from inside the scatter was measured slower than
// the separate histogram launch: device-scope atomics cost ~8 us per pass.)
#include <atomic>

#include "kernels.h"

namespace lshmoe {

namespace {

constexpr int kSortThreads = 256;
// A sort tile holds TILE keys (kSortTile = 2048 unless the plan picks a smaller one for small inputs, so that
// more workgroups share the work): TILE / 256 keys per thread, TILE / 64 wave-sized groups whose per-bin
// counts form a row of TILE / 64 + 1 words (padded against bank conflicts) in LDS.
constexpr int kTableBatch = 32;                        // count-table rows a thread fetches per round trip
constexpr int kSegThreads = 256;
constexpr int kSegItems = kSegTile / kSegThreads;     // 4
constexpr int kSegTileBits = 10;
static_assert((1 << kSegTileBits) == kSegTile, "kSegTileBits");

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
    // bbits <= 63; ids with bits above bbits violate the contract too and must not reach the expert field
    key = ((uint64_t)e << src.bbits) | (src.bucket[i / src.k] & ((1ull << src.bbits) - 1ull));
    idx = (int32_t)i;
  } else {
    key = src.key[i];
    idx = src.idx[i];
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
  for (int w = 0; w < 256 / kWave; ++w) {
    if (w < wave) before += wave_sum[w];
    total += wave_sum[w];
  }
  __syncthreads();
  return before + inc - v;
}

// Tile histogram of one pass.  FUSED: row `tile` of a tile-major table.  Otherwise: column `tile` of a
// bin-major table (scanned next).
template <bool FIRST, bool FUSED, int TILE = kSortTile>
__global__ __launch_bounds__(kSortThreads) void sort_hist_kernel(KeySource src, uint32_t N, int shift, uint32_t mask,
                                                                 uint32_t nblk, uint32_t* __restrict__ table,
                                                                 uint32_t* __restrict__ clear = nullptr,
                                                                 uint32_t clear_n = 0) {
  constexpr int kSortItems = TILE / kSortThreads;
  __shared__ uint32_t h[kGroupBins];
  if (clear != nullptr && blockIdx.x * kSortThreads + threadIdx.x < clear_n)  // counters a later kernel adds to
    clear[blockIdx.x * kSortThreads + threadIdx.x] = 0;
  h[threadIdx.x] = 0;
  h[threadIdx.x + 256] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * TILE;
  uint64_t key[kSortItems];
  int32_t idx[kSortItems];
#pragma unroll
  for (int it = 0; it < kSortItems; ++it)
    load_item<FIRST>(src, min(base + it * kSortThreads + threadIdx.x, N - 1), key[it], idx[it]);
#pragma unroll
  for (int it = 0; it < kSortItems; ++it)
    if (base + it * kSortThreads + threadIdx.x < N) atomicAdd(&h[(uint32_t)(key[it] >> shift) & mask], 1u);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const uint32_t bin = threadIdx.x + 256 * j;
    if (FUSED) {
      table[blockIdx.x * kGroupBins + bin] = h[bin];
    } else if (bin <= mask) {
      table[bin * nblk + blockIdx.x] = h[bin];  // bin-major: a scan over the table orders by (bin, tile)
    }
  }
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

constexpr int kBinChunk = 2048;  // most-significant-digit route: keys one workgroup sorts (see bin_sort_kernel)

// The chunk table: written by block 0 of the global scatter from the bins' sizes.
__device__ __forceinline__ void write_chunk_table(uint32_t total0, uint32_t total1, uint32_t* bin_start,
                                                  uint32_t* chunk_tbl, uint32_t* wave_sum) {
  const uint32_t c0 = (total0 + kBinChunk - 1) / kBinChunk, c1 = (total1 + kBinChunk - 1) / kBinChunk;
  uint32_t half, rest;
  const uint32_t at0 = block_exclusive_scan(c0, wave_sum, half);
  const uint32_t at1 = half + block_exclusive_scan(c1, wave_sum, rest);
  for (uint32_t j = 0; j < c0; ++j) chunk_tbl[at0 + j] = (threadIdx.x << 16) | j;
  for (uint32_t j = 0; j < c1; ++j) chunk_tbl[at1 + j] = ((threadIdx.x + 256u) << 16) | j;
  const int several = __syncthreads_or(c0 > 1 || c1 > 1);
  if (threadIdx.x == 0) {
    bin_start[kGroupBins + 1] = half + rest;
    bin_start[kGroupBins + 2] = several ? 1u : 0u;
  }
}

struct PassArgs {
  int shift;            // this pass's digit is (key >> shift) & mask
  uint32_t mask;
  uint32_t nblk;
  const uint32_t* table;  // FUSED: tile-major counts of this pass; else the scanned bin-major offsets
  uint32_t* bin_start;    // FUSED, optional: block 0 writes the first output position of every bin, then N,
  uint32_t* chunk_tbl;    // then the number of chunks and whether a bin has several; and the chunk table
};

template <bool FIRST, bool FUSED, int TILE = kSortTile>
__global__ __launch_bounds__(kSortThreads) void sort_scatter_kernel(KeySource src, uint32_t N, PassArgs a,
                                                                    uint64_t* __restrict__ dst_key,
                                                                    int32_t* __restrict__ dst_idx) {
  constexpr int kSortItems = TILE / kSortThreads, kGroupsPerTile = TILE / kWave, kGhStride = kGroupsPerTile + 1;
  extern __shared__ uint32_t gh[];  // [kGroupBins][kGhStride] per-bin counts of each 64-key group, then start offsets
  __shared__ uint32_t wave_sum[4];
  __shared__ uint32_t part[2][2][kGroupBins];  // FUSED: [before/total][tile parity][bin]
  const uint32_t base = blockIdx.x * TILE;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  uint64_t key[kSortItems];
  int32_t idx[kSortItems];
  uint32_t rank[kSortItems];
  // all of the tile's loads are issued before the first use (positions past N re-read the last key and are
  // masked out below), so the tile costs one memory round trip
#pragma unroll
  for (int it = 0; it < kSortItems; ++it)
    load_item<FIRST>(src, min(base + it * kSortThreads + threadIdx.x, N - 1), key[it], idx[it]);
  static_assert((kGroupBins * kGhStride) % 4 == 0, "gh is cleared 16 bytes at a time");
  for (int i = threadIdx.x; i < kGroupBins * kGhStride / 4; i += kSortThreads)  // while the loads fly
    reinterpret_cast<uint4*>(gh)[i] = make_uint4(0, 0, 0, 0);
  if (FUSED) {
    // counts[tile][bin]: keys of bin b in earlier tiles come first, after all keys of smaller bins
    // Threads 0..127 walk the even tiles' rows, threads 128..255 the odd ones, four bins (16 bytes) each,
    // in batches of independent loads; the two parities are then combined through LDS.
    {
      const uint32_t parity = threadIdx.x >> 7, b4 = (threadIdx.x & 127) * 4;
      uint32_t bef[4] = {0, 0, 0, 0}, tot[4] = {0, 0, 0, 0};
      for (uint32_t t0 = parity; t0 < a.nblk; t0 += 2 * kTableBatch) {
        uint4 v[kTableBatch];
#pragma unroll
        for (int q = 0; q < kTableBatch; ++q) {
          const uint32_t t = t0 + 2 * q;
          v[q] = t < a.nblk ? *reinterpret_cast<const uint4*>(a.table + t * kGroupBins + b4) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < kTableBatch; ++q) {
          const bool earlier = t0 + 2 * q < blockIdx.x;
          const uint32_t w[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            tot[j] += w[j];
            bef[j] += earlier ? w[j] : 0u;
          }
        }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        part[0][parity][b4 + j] = bef[j];
        part[1][parity][b4 + j] = tot[j];
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kSortItems; ++it) {
    const uint32_t i = base + it * kSortThreads + threadIdx.x;
    const bool valid = i < N;
    const uint32_t digit = (uint32_t)(key[it] >> a.shift) & a.mask;
    uint64_t same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < kMaxDigitBits; ++b) {
      const bool bit = (digit >> b) & 1u;
      const uint64_t bal = __ballot(bit);
      same &= bit ? bal : ~bal;
    }
    rank[it] = (uint32_t)__popcll(same & lt_mask);
    if (valid && rank[it] == 0) gh[digit * kGhStride + it * (kSortThreads / kWave) + wave] = (uint32_t)__popcll(same);
  }

  // first output position of each bin for this tile
  uint32_t start[2];
  if (FUSED) {
    __syncthreads();
    uint32_t before[2], total[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t bin = threadIdx.x + 256 * j;
      before[j] = part[0][0][bin] + part[0][1][bin];
      total[j] = part[1][0][bin] + part[1][1][bin];
    }
    uint32_t half;  // keys in bins 0..255
    start[0] = block_exclusive_scan(total[0], wave_sum, half) + before[0];
    uint32_t unused;
    start[1] = half + block_exclusive_scan(total[1], wave_sum, unused) + before[1];
    if (a.bin_start != nullptr && blockIdx.x == 0) {  // nothing comes before tile 0: its starts are the bins' starts
      a.bin_start[threadIdx.x] = start[0];
      a.bin_start[threadIdx.x + 256] = start[1];
      if (threadIdx.x == 0) a.bin_start[kGroupBins] = N;
      write_chunk_table(total[0], total[1], a.bin_start, a.chunk_tbl, wave_sum);
    }
  } else {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t bin = threadIdx.x + 256 * j;
      start[j] = bin <= a.mask ? a.table[bin * a.nblk + blockIdx.x] : 0;
    }
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {  // counts -> start offsets along the bin's row (independent reads, then register adds)
    uint32_t* row = gh + (threadIdx.x + 256 * j) * kGhStride;
    uint32_t c[kGroupsPerTile];
#pragma unroll
    for (int g = 0; g < kGroupsPerTile; ++g) c[g] = row[g];
    uint32_t run = start[j];
#pragma unroll
    for (int g = 0; g < kGroupsPerTile; ++g) {
      row[g] = run;
      run += c[g];
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kSortItems; ++it) {
    const uint32_t i = base + it * kSortThreads + threadIdx.x;
    if (i < N) {
      const uint32_t digit = (uint32_t)(key[it] >> a.shift) & a.mask;
      const uint32_t pos = gh[digit * kGhStride + it * (kSortThreads / kWave) + wave] + rank[it];
      dst_key[pos] = key[it];
      dst_idx[pos] = idx[it];
    }
  }
}

// Head flags of kSegItems consecutive sorted positions starting at `base`: position p starts a cluster when
// its key differs from the key before it.  The keys are fetched up front (indices clamped into range).
__device__ __forceinline__ void load_heads(const uint64_t* __restrict__ key, uint32_t base, uint32_t N,
                                           uint64_t (&kv)[kSegItems + 1], bool (&head)[kSegItems]) {
#pragma unroll
  for (int it = 0; it <= kSegItems; ++it) {
    const uint32_t p = base + it;  // kv[it] is the key at position p - 1
    kv[it] = key[min(p == 0 ? 0u : p - 1, N - 1)];
  }
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) {
    const uint32_t p = base + it;
    head[it] = p < N && (p == 0 || kv[it + 1] != kv[it]);
  }
}

// Also clears the centroid step's window counters (each tile clears those of its own positions).
__global__ __launch_bounds__(kSegThreads) void seg_count_kernel(const uint64_t* __restrict__ key, uint32_t N,
                                                                uint32_t nblk, uint32_t* __restrict__ blocksum,
                                                                uint32_t* __restrict__ window_counters) {
  __shared__ uint32_t wave_sum[kSegThreads / kWave];
  constexpr uint32_t kCountersPerTile = 2 * kSegTile / kCentroidWindow;
  static_assert(kSegTile % kCentroidWindow == 0 && kCountersPerTile <= kSegThreads, "window counters per tile");
  if (threadIdx.x < kCountersPerTile) window_counters[blockIdx.x * kCountersPerTile + threadIdx.x] = 0;
  const uint32_t base = blockIdx.x * kSegTile + threadIdx.x * kSegItems;
  uint64_t kv[kSegItems + 1];
  bool head[kSegItems];
  load_heads(key, base, N, kv, head);
  uint32_t c = 0;
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) c += head[it] ? 1u : 0u;
  uint32_t total;
  block_exclusive_scan(c, wave_sum, total);
  if (threadIdx.x == 0) {
    blocksum[blockIdx.x] = total;
    if (blockIdx.x == 0) blocksum[nblk] = 0;  // after a scan this slot holds the grand total
  }
}

// SELF_PREFIX: blocksum holds per-tile head counts and the block adds up the tiles before it itself;
// otherwise blocksum has been scanned.
template <bool SELF_PREFIX>
__global__ __launch_bounds__(kSegThreads) void seg_write_kernel(
    const uint64_t* __restrict__ key, const int32_t* __restrict__ perm, uint32_t N, uint32_t E, int bbits,
    const uint32_t* __restrict__ blocksum, int32_t* __restrict__ seg_offsets, int32_t* __restrict__ seg_expert,
    int32_t* __restrict__ expert_offsets, int32_t* __restrict__ seg_of, int32_t* __restrict__ num_segments,
    uint32_t* __restrict__ window_counters = nullptr, const uint4* __restrict__ chunk_heads = nullptr,
    const uint32_t* __restrict__ chunk_count = nullptr) {
  __shared__ uint32_t wave_sum[kSegThreads / kWave];
  constexpr uint32_t kCountersPerTile = 2 * kSegTile / kCentroidWindow;
  if (window_counters != nullptr && threadIdx.x < kCountersPerTile)  // when no seg_count_kernel ran to clear them
    window_counters[blockIdx.x * kCountersPerTile + threadIdx.x] = 0;
  uint32_t tiles_before = 0;
  if (SELF_PREFIX) {
    uint32_t part = 0;
    for (uint32_t t = threadIdx.x; t < blockIdx.x; t += kSegThreads) part += blocksum[t];
    if (chunk_heads != nullptr) {
      // heads of bins sorted as one chunk come per chunk: {first tile, heads in that tile and the next two}
      const uint32_t nch = *chunk_count;
      for (uint32_t c = threadIdx.x; c < nch; c += kSegThreads) {
        const uint4 v = chunk_heads[c];
        part += (v.x < blockIdx.x ? v.y : 0u) + (v.x + 1 < blockIdx.x ? v.z : 0u) + (v.x + 2 < blockIdx.x ? v.w : 0u);
      }
    }
    block_exclusive_scan(part, wave_sum, tiles_before);
  } else {
    tiles_before = blocksum[blockIdx.x];
  }
  const uint32_t base = blockIdx.x * kSegTile + threadIdx.x * kSegItems;
  uint64_t kv[kSegItems + 1];
  bool head[kSegItems];
  load_heads(key, base, N, kv, head);
  int32_t a[kSegItems];
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) a[it] = perm[min(base + it, N - 1)];
  uint32_t c = 0;
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) c += head[it] ? 1u : 0u;
  uint32_t total;
  uint32_t seg = tiles_before + block_exclusive_scan(c, wave_sum, total);  // heads before this thread
#pragma unroll
  for (int it = 0; it < kSegItems; ++it) {
    const uint32_t p = base + it;
    if (p >= N) break;
    const uint32_t e = (uint32_t)(kv[it + 1] >> bbits);
    if (head[it]) {
      seg_offsets[seg] = (int32_t)p;
      seg_expert[seg] = (int32_t)e;
      const uint32_t first = p == 0 ? 0u : (uint32_t)(kv[it] >> bbits) + 1u;
      for (uint32_t x = first; x <= e; ++x) expert_offsets[x] = (int32_t)seg;  // experts that start (or are empty) here
      ++seg;
    }
    seg_of[a[it]] = (int32_t)(seg - 1);
    if (p == N - 1) {
      for (uint32_t x = e + 1; x <= E; ++x) expert_offsets[x] = (int32_t)seg;
      seg_offsets[seg] = (int32_t)N;
      *num_segments = (int32_t)seg;
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Tiny inputs (N <= kSmallMaxN): the whole grouping in ONE workgroup of 16 waves and one launch.  With a
// few thousand keys every multi-launch scheme is dominated by launch and drain latency (~4 us per kernel)
// and one compute unit sorts them faster than the launches alone would take (measured: 24 us instead of
// 38 us for compress at N = 2048; from about 16k keys on the single compute unit is the slower route).
// Each wave owns a contiguous slice of the array.  Per pass: count digits per (wave, bin) with LDS atomics,
// turn the counts into start offsets in (bin, wave) order, then walk the slice again 64 keys at a time:
// a key's position is the running offset of its (wave, bin) plus its rank among the equal digits of its
// round (wave ballots).  Slices and rounds follow element order, so the sort is stable.
struct SmallArgs {
  int passes, bbits;
  int shift[8], width[8];
  uint32_t N, E;
  uint64_t* keybuf[2];
  int32_t* idxbuf[2];
  int32_t *seg_offsets, *seg_expert, *expert_offsets, *perm, *seg_of, *num_segments;
  uint32_t* window_counters;  // cleared here for the centroid step
};

constexpr int kSmallWaves = 16;

__device__ __forceinline__ uint32_t block_exclusive_scan_1024(uint32_t v, uint32_t* wave_sum /*[16]*/, uint32_t& total) {
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
  for (int w = 0; w < kSmallWaves; ++w) {
    if (w < wave) before += wave_sum[w];
    total += wave_sum[w];
  }
  __syncthreads();
  return before + inc - v;
}

__global__ __launch_bounds__(kSmallWaves * 64) void small_group_kernel(KeySource src, SmallArgs a) {
  __shared__ uint32_t cnt[kSmallWaves][kGroupBins];  // 32 KB
  __shared__ uint32_t wave_sum[kSmallWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const uint32_t N = a.N;
  if (threadIdx.x < 2 * ((N + kCentroidWindow - 1) / kCentroidWindow)) a.window_counters[threadIdx.x] = 0;
  const uint32_t slice = ((N + kSmallWaves - 1) / kSmallWaves + 63u) & ~63u;  // keys per wave, whole rounds
  const uint32_t lo = min((uint32_t)wave * slice, N), hi = min(lo + slice, N);

  for (int p = 0; p < a.passes; ++p) {
    const bool first = p == 0, last = p == a.passes - 1;
    const int shift = a.shift[p];
    const uint32_t mask = (1u << a.width[p]) - 1u;
    KeySource from = src;
    from.key = a.keybuf[(p + 1) & 1];
    from.idx = a.idxbuf[(p + 1) & 1];
    uint64_t* dkey = a.keybuf[p & 1];
    int32_t* didx = last ? a.perm : a.idxbuf[p & 1];
    auto load = [&](uint32_t i, uint64_t& key, int32_t& idx) {
      if (first) load_item<true>(from, i, key, idx);
      else load_item<false>(from, i, key, idx);
    };

    for (int i = threadIdx.x; i < kSmallWaves * kGroupBins; i += kSmallWaves * 64) (&cnt[0][0])[i] = 0;
    __syncthreads();
    for (uint32_t base = lo; base < hi; base += 256) {  // four rounds of loads in flight
      uint64_t key[4];
      int32_t idx[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) load(min(base + q * 64 + lane, N - 1), key[q], idx[q]);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (base + q * 64 + lane < hi) atomicAdd(&cnt[wave][(uint32_t)(key[q] >> shift) & mask], 1u);
    }
    __syncthreads();
    {  // counts -> start offsets, ordered by (bin, wave)
      uint32_t c[kSmallWaves], tot = 0;
      const bool owner = threadIdx.x < kGroupBins;
#pragma unroll
      for (int w = 0; w < kSmallWaves; ++w) {
        c[w] = owner ? cnt[w][threadIdx.x] : 0u;
        tot += c[w];
      }
      uint32_t unused;
      uint32_t run = block_exclusive_scan_1024(tot, wave_sum, unused);
      if (owner) {
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) {
          cnt[w][threadIdx.x] = run;
          run += c[w];
        }
      }
    }
    __syncthreads();
    {
      uint64_t key;
      int32_t idx;
      if (lo < hi) load(min(lo + lane, N - 1), key, idx);
      for (uint32_t base = lo; base < hi; base += 64) {
        uint64_t nkey = 0;
        int32_t nidx = 0;
        if (base + 64 < hi) load(min(base + 64 + lane, N - 1), nkey, nidx);  // next round's keys fly meanwhile
        const bool valid = base + lane < hi;
        const uint32_t digit = (uint32_t)(key >> shift) & mask;
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kMaxDigitBits; ++b) {
          const bool bit = (digit >> b) & 1u;
          const uint64_t bal = __ballot(bit);
          same &= bit ? bal : ~bal;
        }
        const uint32_t rank = (uint32_t)__popcll(same & lt_mask);
        const uint32_t start = cnt[wave][digit];
        if (valid) {
          dkey[start + rank] = key;
          didx[start + rank] = idx;
          if (rank == 0) cnt[wave][digit] = start + (uint32_t)__popcll(same);  // after every lane of the round has read
        }
        key = nkey;
        idx = nidx;
      }
    }
    __syncthreads();  // the pass's global writes are visible to the whole workgroup (one compute unit, one L1)
  }

  // number the clusters: head flags over the sorted keys
  const uint64_t* skey = a.keybuf[(a.passes - 1) & 1];
  uint32_t heads = 0;
  for (uint32_t base = lo; base < hi; base += 64) {
    const uint32_t i = base + lane;
    const bool head = i < hi && (i == 0 || skey[i] != skey[i - 1]);
    heads += (uint32_t)__popcll(__ballot(head));
  }
  uint32_t total;
  uint32_t seg_base = block_exclusive_scan_1024(lane == 0 ? heads : 0u, wave_sum, total);
  seg_base = (uint32_t)__shfl((int)seg_base, 0, 64);  // lane 0 holds the heads before this wave's slice
  for (uint32_t base = lo; base < hi; base += 64) {
    const uint32_t i = base + lane;
    const bool valid = i < hi;
    const uint32_t ic = min(i, N - 1);  // lanes past the slice re-read a valid key (ic - 1 must not wrap when N == 1)
    const uint64_t kcur = skey[ic], kprev = skey[ic == 0 ? 0u : ic - 1u];
    const bool head = valid && (i == 0 || kcur != kprev);
    const uint64_t hmask = __ballot(head);
    const uint32_t seg = seg_base + (uint32_t)__popcll(hmask & (lt_mask | (1ull << lane))) - 1u;  // heads up to and including i
    if (valid) {
      const uint32_t e = (uint32_t)(kcur >> a.bbits);
      if (head) {
        a.seg_offsets[seg] = (int32_t)i;
        a.seg_expert[seg] = (int32_t)e;
        const uint32_t from_e = i == 0 ? 0u : (uint32_t)(kprev >> a.bbits) + 1u;
        for (uint32_t x = from_e; x <= e; ++x) a.expert_offsets[x] = (int32_t)seg;  // experts that start (or are empty) here
      }
      a.seg_of[a.perm[i]] = (int32_t)seg;
      if (i == N - 1) {
        for (uint32_t x = e + 1; x <= a.E; ++x) a.expert_offsets[x] = (int32_t)(seg + 1);
        a.seg_offsets[seg + 1] = (int32_t)N;
        *a.num_segments = (int32_t)(seg + 1);
      }
    }
    seg_base += (uint32_t)__popcll(hmask);
  }
}

// ---------------------------------------------------------------------------------------------------
// Most-significant-digit route (up to kFusedMaxTiles tiles): ONE global pass on the top digit of the key
// splits the assignments into up to 512 bins (stable, so a bin keeps ascending assignment order).  A bin
// is cut into chunks of at most kBinChunk consecutive keys; one workgroup sorts one chunk on the remaining
// key bits inside LDS; a bin of several chunks is then merged by rank.  That replaces a histogram and a
// scatter launch per further digit by one launch (two when some bin has more than kBinChunk keys).
//
// Chunk sort, two ways:
//   up to kBinFast keys and no crowded sub-bin: the keys are thrown into sub-bins by their next (up to) 8
//     bits with LDS counters, in whatever order they arrive; a key's rank is the start of its sub-bin plus
//     the number of keys of that sub-bin that come before it, by key and, among equal keys, by place in the
//     chunk (stable).  Only keys that agree in those 8 bits are compared: a handful.
//   otherwise: least-significant-digit radix passes between two LDS buffers (each wave owns a slice of the
//     chunk; counts per (wave, digit); ranks inside a round of 64 keys from wave ballots), the last pass
//     writing to global memory.  Its cost does not depend on how many keys are equal.
struct BinSortArgs {
  const uint32_t* bin_start;  // [bins + 1], then [bins + 1] = number of chunks, [bins + 2] = 1 if a bin has several
  const uint32_t* chunk_tbl;  // chunk w is chunk (entry & 0xffff) of bin (entry >> 16)
  uint64_t* key[2];           // [0]: keys after the global pass; [1]: receives the sorted keys
  int32_t* idx[2];            // [0]: assignment ids after the global pass
  int32_t* perm;              // receives the sorted assignment ids
  int passes;                 // radix passes over the low key bits
  int shift[8], width[8];     // their digits, least significant first
  int sub_shift;              // sub-bin of a key is (key >> sub_shift) & sub_mask
  uint32_t sub_mask;
  uint32_t* tile_heads;       // [tiles of kSegTile positions]: cluster heads per tile of bins of several chunks (atomics)
  uint4* chunk_heads;         // [chunks]: {first tile, heads in it, in the next, in the one after} of a bin of one chunk
};

// Publishes the heads counted in LDS per numbering tile (a chunk's positions touch at most kChunkTiles of them)
// as the chunk's own record: plain stores, no contention (hundreds of workgroups adding to a handful of per-tile
// counters cost several microseconds on small inputs).  Every thread of the workgroup calls it.
constexpr int kChunkTiles = kBinChunk / kSegTile + 1;
static_assert(kChunkTiles == 3, "a chunk record holds three tile counts");
__device__ __forceinline__ void publish_chunk_heads(const uint32_t* tile_cnt, uint32_t first_tile, uint4* record) {
  __syncthreads();
  if (threadIdx.x == 0) *record = make_uint4(first_tile, tile_cnt[0], tile_cnt[1], tile_cnt[2]);
}

constexpr int kBinFast = 1024;                     // up to here the sub-bin way is tried first
constexpr int kBinWaves = 4;
constexpr int kBinThreads = kBinWaves * 64;
constexpr int kBinItems = kBinFast / kBinThreads;  // keys per thread on the sub-bin way
constexpr int kSubBins = 256;
constexpr uint32_t kSubBinCrowd = 32;              // a sub-bin with more keys sends the chunk the radix way
constexpr size_t kBinSortLds = 2 * (size_t)kBinChunk * (8 + 4);  // two (key, id) buffers: 48 KB

__global__ __launch_bounds__(kBinThreads) void bin_sort_kernel(BinSortArgs a) {
  extern __shared__ uint64_t bin_lds[];            // radix way: keys [2][kBinChunk], then ids [2][kBinChunk]
  __shared__ uint32_t cnt[kBinWaves][kGroupBins];  // 8 KB; the sub-bin way keeps its keys here
  __shared__ uint32_t place_s[kBinFast];           // sub-bin way: a key's place in the chunk before sorting
  __shared__ uint32_t sub_cnt[kSubBins], sub_base[kSubBins];
  __shared__ uint32_t wave_sum[kBinWaves];
  __shared__ uint32_t tile_cnt[kChunkTiles];
  if (blockIdx.x >= a.bin_start[kGroupBins + 1]) return;
  if (threadIdx.x < (uint32_t)kChunkTiles) tile_cnt[threadIdx.x] = 0;  // a barrier follows on every way
  const uint32_t entry = a.chunk_tbl[blockIdx.x];
  const uint32_t bin = entry >> 16, chunk = entry & 0xffffu;
  const uint32_t lo_bin = a.bin_start[bin], hi_bin = a.bin_start[bin + 1];
  const uint32_t lo = lo_bin + chunk * kBinChunk, hi = min(lo + (uint32_t)kBinChunk, hi_bin);
  const uint32_t n = hi - lo;
  // a bin of one chunk is finished here; the chunks of a larger bin are sorted in place and merged afterwards
  const bool alone = hi_bin - lo_bin <= (uint32_t)kBinChunk;
  uint64_t* out_key = alone ? a.key[1] : a.key[0];
  int32_t* out_idx = alone ? a.perm : a.idx[0];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  if (n <= (uint32_t)kBinFast) {
    static_assert(sizeof(cnt) >= kBinFast * sizeof(uint64_t), "keys of a small chunk fit in the count table");
    static_assert(kSubBins == kBinThreads, "one sub-bin counter per thread");
    uint64_t* key_s = reinterpret_cast<uint64_t*>(&cnt[0][0]);
    uint64_t key[kBinItems];
    int32_t idx[kBinItems];
    uint32_t sub[kBinItems], slot[kBinItems];
#pragma unroll
    for (int q = 0; q < kBinItems; ++q) {
      const uint32_t i = threadIdx.x + q * kBinThreads;
      key[q] = 0;
      idx[q] = 0;
      if (i < n) {
        key[q] = a.key[0][lo + i];
        idx[q] = a.idx[0][lo + i];
      }
    }
    sub_cnt[threadIdx.x] = 0;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kBinItems; ++q) {
      sub[q] = (uint32_t)(key[q] >> a.sub_shift) & a.sub_mask;
      if (threadIdx.x + q * kBinThreads < n) slot[q] = atomicAdd(&sub_cnt[sub[q]], 1u);
    }
    __syncthreads();
    const uint32_t mine = sub_cnt[threadIdx.x];
    const int crowded = __syncthreads_or(mine > kSubBinCrowd);
    if (!crowded) {
      {
        uint32_t unused;
        sub_base[threadIdx.x] = block_exclusive_scan(mine, wave_sum, unused);
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < kBinItems; ++q) {
        const uint32_t i = threadIdx.x + q * kBinThreads;
        if (i < n) {
          const uint32_t at = sub_base[sub[q]] + slot[q];
          key_s[at] = key[q];
          place_s[at] = i;
        }
      }
      __syncthreads();  // also: every key of the chunk has been read before the first one is written back
#pragma unroll
      for (int q = 0; q < kBinItems; ++q) {
        const uint32_t i = threadIdx.x + q * kBinThreads;
        if (i < n) {
          const uint32_t first = sub_base[sub[q]], m = sub_cnt[sub[q]];
          uint32_t rank = first;
          bool repeat = false;  // an equal key comes before this one: not the head of its cluster
          for (uint32_t t = 0; t < m; ++t) {
            const uint64_t kj = key_s[first + t];
            const uint32_t pj = place_s[first + t];
            const bool eq_before = kj == key[q] && pj < i;
            repeat |= eq_before;
            rank += (kj < key[q] || eq_before) ? 1u : 0u;
          }
          out_key[lo + rank] = key[q];
          out_idx[lo + rank] = idx[q];
          if (alone && !repeat) atomicAdd(&tile_cnt[((lo + rank) >> kSegTileBits) - (lo >> kSegTileBits)], 1u);
        }
      }
      publish_chunk_heads(tile_cnt, lo >> kSegTileBits, a.chunk_heads + blockIdx.x);  // zeros unless alone
      return;
    }
    __syncthreads();  // the radix way below reuses cnt
  }

  // radix way: the chunk lives in LDS between the passes
  uint64_t* const kbuf = bin_lds;                                            // [2][kBinChunk]
  int32_t* const ibuf = reinterpret_cast<int32_t*>(bin_lds + 2 * kBinChunk);  // [2][kBinChunk]
  for (uint32_t i = threadIdx.x; i < n; i += kBinThreads) {
    kbuf[i] = a.key[0][lo + i];
    ibuf[i] = a.idx[0][lo + i];
  }
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const uint32_t slice = ((n + kBinWaves - 1) / kBinWaves + 63u) & ~63u;  // keys per wave, whole rounds
  const uint32_t wlo = min((uint32_t)wave * slice, n), whi = min(wlo + slice, n);
  for (int p = 0; p < a.passes; ++p) {
    const int shift = a.shift[p];
    const uint32_t mask = (1u << a.width[p]) - 1u;
    const uint64_t* skey = kbuf + (p & 1) * kBinChunk;
    const int32_t* sidx = ibuf + (p & 1) * kBinChunk;
    uint64_t* dkey = kbuf + ((p + 1) & 1) * kBinChunk;
    int32_t* didx = ibuf + ((p + 1) & 1) * kBinChunk;
    for (int i = threadIdx.x; i < kBinWaves * kGroupBins; i += kBinThreads) (&cnt[0][0])[i] = 0;
    __syncthreads();  // also: the chunk (first pass) or the previous pass's output is in LDS
    for (uint32_t i = wlo + lane; i < whi; i += 64) atomicAdd(&cnt[wave][(uint32_t)(skey[i] >> shift) & mask], 1u);
    __syncthreads();
    {  // counts -> start offsets, ordered by (digit, wave); two digits per thread
      uint32_t c[2][kBinWaves], tot[2] = {0, 0};
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int w = 0; w < kBinWaves; ++w) {
          c[j][w] = cnt[w][threadIdx.x + 256 * j];
          tot[j] += c[j][w];
        }
      uint32_t half, unused;
      uint32_t run0 = block_exclusive_scan(tot[0], wave_sum, half);
      uint32_t run1 = half + block_exclusive_scan(tot[1], wave_sum, unused);
#pragma unroll
      for (int w = 0; w < kBinWaves; ++w) {
        cnt[w][threadIdx.x] = run0;
        run0 += c[0][w];
        cnt[w][threadIdx.x + 256] = run1;
        run1 += c[1][w];
      }
    }
    __syncthreads();
    for (uint32_t base = wlo; base < whi; base += 64) {
      const bool valid = base + lane < whi;
      const uint32_t at = min(base + lane, n - 1);
      const uint64_t key = skey[at];
      const int32_t idx = sidx[at];
      const uint32_t digit = (uint32_t)(key >> shift) & mask;
      uint64_t same = __ballot(valid);
#pragma unroll
      for (int b = 0; b < kMaxDigitBits; ++b) {
        const bool bit = (digit >> b) & 1u;
        const uint64_t bal = __ballot(bit);
        same &= bit ? bal : ~bal;
      }
      const uint32_t rank = (uint32_t)__popcll(same & lt_mask);
      const uint32_t start = cnt[wave][digit];
      if (valid) {
        dkey[start + rank] = key;
        didx[start + rank] = idx;
        if (rank == 0) cnt[wave][digit] = start + (uint32_t)__popcll(same);  // after every lane of the round has read
      }
    }
    __syncthreads();
  }
  // the sorted chunk is in LDS: write it out in order and count the cluster heads
  const uint64_t* fkey = kbuf + (a.passes & 1) * kBinChunk;
  const int32_t* fidx = ibuf + (a.passes & 1) * kBinChunk;
  for (uint32_t i = threadIdx.x; i < n; i += kBinThreads) {
    const uint64_t k = fkey[i];
    out_key[lo + i] = k;
    out_idx[lo + i] = fidx[i];
    if (alone && (i == 0 || fkey[i - 1] != k)) atomicAdd(&tile_cnt[((lo + i) >> kSegTileBits) - (lo >> kSegTileBits)], 1u);
  }
  publish_chunk_heads(tile_cnt, lo >> kSegTileBits, a.chunk_heads + blockIdx.x);  // zeros unless alone
}

// Merge of the sorted chunks of a bin that has several: the final place of a key is the bin's start plus
// its place in its own chunk plus, for every other chunk of the bin, the number of keys there that come
// before it: the smaller ones, and for an earlier chunk also the equal ones (chunks follow assignment
// order, so this keeps the sort stable).  One workgroup per chunk; the other chunks pass through LDS one
// at a time and are searched by bisection; kMergeSlices workgroups share the keys of one chunk, so that a
// bin holding most of the input still spreads over the chip.  Leaves at once when no bin has several chunks.
constexpr int kMergeSlices = 4;  // workgroups that share the keys of one chunk
constexpr int kMergeOwn = kBinChunk / kMergeSlices / kBinThreads;  // keys per thread: 2

__global__ __launch_bounds__(kBinThreads) void bin_merge_kernel(BinSortArgs a) {
  __shared__ uint64_t other[kBinChunk];  // 16 KB
  if (a.bin_start[kGroupBins + 2] == 0) return;   // no bin has several chunks: the usual case
  // a fixed, small grid walks the (chunk, slice) items: the launch is idle on almost every input, and an idle
  // launch of one workgroup per item costs 2 us more than this one
  const uint32_t items = a.bin_start[kGroupBins + 1] * kMergeSlices;
  for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
  const uint32_t cidx = item / kMergeSlices, slice = item % kMergeSlices;
  const uint32_t entry = a.chunk_tbl[cidx];
  const uint32_t bin = entry >> 16, chunk = entry & 0xffffu;
  const uint32_t lo_bin = a.bin_start[bin], hi_bin = a.bin_start[bin + 1];
  if (hi_bin - lo_bin <= (uint32_t)kBinChunk) continue;   // workgroup-uniform
  const uint32_t chunks = (hi_bin - lo_bin + kBinChunk - 1) / kBinChunk;
  const uint32_t lo = lo_bin + chunk * kBinChunk, hi = min(lo + (uint32_t)kBinChunk, hi_bin);
  const uint32_t n = hi - lo;
  constexpr int kItems = kBinChunk / kBinThreads;  // keys of another chunk a thread stages: 8
  uint64_t key[kMergeOwn];
  uint32_t before[kMergeOwn];
  bool repeat[kMergeOwn];
#pragma unroll
  for (int q = 0; q < kMergeOwn; ++q) {
    const uint32_t i = slice * (kBinChunk / kMergeSlices) + threadIdx.x + q * kBinThreads;
    key[q] = i < n ? a.key[0][lo + i] : 0;
    before[q] = i;  // keys before it in its own chunk
    repeat[q] = i < n && i > 0 && a.key[0][lo + i - 1] == key[q];
  }
  // the other chunks pass through LDS one at a time; the next one is fetched into registers while the
  // current one is searched
  auto fetch = [&](uint32_t c, uint64_t (&v)[kItems]) {
    const uint32_t olo = lo_bin + c * kBinChunk, on = min((uint32_t)kBinChunk, hi_bin - olo);
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
      const uint32_t i = threadIdx.x + q * kBinThreads;
      v[q] = a.key[0][olo + min(i, on - 1)];
    }
  };
  auto next_other = [&](uint32_t c) { return c + 1 == chunk ? c + 2 : c + 1; };
  uint64_t staged[kItems];
  uint32_t c = chunk == 0 ? 1u : 0u;
  fetch(c, staged);
  for (; c < chunks; c = next_other(c)) {
    const uint32_t on = min((uint32_t)kBinChunk, hi_bin - (lo_bin + c * kBinChunk));
    __syncthreads();  // the previous chunk has been searched
#pragma unroll
    for (int q = 0; q < kItems; ++q) other[threadIdx.x + q * kBinThreads] = staged[q];
    __syncthreads();
    if (next_other(c) < chunks) fetch(next_other(c), staged);
    const bool earlier = c < chunk;
    // number of keys of the other chunk that are < key (later chunk) or <= key (earlier chunk): bisection
    // with a fixed number of steps, the thread's keys side by side so that the LDS reads overlap
    uint32_t pos[kMergeOwn];
#pragma unroll
    for (int q = 0; q < kMergeOwn; ++q) pos[q] = 0;
    for (uint32_t step = kBinChunk; step >= 1; step >>= 1) {
#pragma unroll
      for (int q = 0; q < kMergeOwn; ++q) {
        const uint32_t t = pos[q] + step;
        const uint64_t v = other[min(t, on) - 1];
        const bool take = t <= on && (earlier ? v <= key[q] : v < key[q]);
        pos[q] = take ? t : pos[q];
      }
    }
#pragma unroll
    for (int q = 0; q < kMergeOwn; ++q) {
      before[q] += pos[q];
      if (earlier && pos[q] > 0 && other[pos[q] - 1] == key[q]) repeat[q] = true;  // an equal key in an earlier chunk
    }
  }
  // the keys land anywhere in the bin: heads are counted per numbering tile in LDS first
  __syncthreads();
  uint32_t* tile_cnt = reinterpret_cast<uint32_t*>(other);
  const uint32_t first_tile = lo_bin >> kSegTileBits, tiles = ((hi_bin - 1) >> kSegTileBits) - first_tile + 1;
  static_assert(sizeof(other) >= (kFusedMaxTiles * kSortTile / kSegTile) * sizeof(uint32_t), "tile counters fit");
  for (uint32_t t = threadIdx.x; t < tiles; t += kBinThreads) tile_cnt[t] = 0;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < kMergeOwn; ++q) {
    const uint32_t i = slice * (kBinChunk / kMergeSlices) + threadIdx.x + q * kBinThreads;
    if (i < n) {
      const uint32_t at = lo_bin + before[q];
      a.key[1][at] = key[q];
      a.perm[at] = a.idx[0][lo + i];
      if (!repeat[q]) atomicAdd(&tile_cnt[(at >> kSegTileBits) - first_tile], 1u);
    }
  }
  __syncthreads();
  for (uint32_t t = threadIdx.x; t < tiles; t += kBinThreads)
    if (tile_cnt[t] != 0) atomicAdd(&a.tile_heads[first_tile + t], tile_cnt[t]);
  __syncthreads();   // `other` is free for the next item
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

template <bool FIRST, bool FUSED, int TILE = kSortTile>
hipError_t launch_scatter(const KeySource& src, uint32_t N, const PassArgs& a, uint64_t* dkey, int32_t* didx,
                          hipStream_t stream) {
  constexpr size_t kScatterLds = (size_t)kGroupBins * (TILE / kWave + 1) * 4;  // 66 KB for tiles of 2048
  auto kern = sort_scatter_kernel<FIRST, FUSED, TILE>;
  static std::atomic<bool> raised{false};  // set once per kernel; repeating the call is harmless
  if (!raised.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kScatterLds);
    if (e != hipSuccess) return e;
    raised.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(kern, dim3(a.nblk), dim3(kSortThreads), kScatterLds, stream, src, N, a, dkey, didx);
  return hipGetLastError();
}

}  // namespace

bool plan_group(int64_t T, int d, int k, int E, int L, int r, GroupPlan* plan) {
  uint64_t nb = 1;  // (2r)^L, known to be < 2^63 by the caller's check
  for (int l = 0; l < L; ++l) nb *= (uint64_t)(2 * r);
  GroupPlan p{};
  p.N = T * k;
  p.ebits = bits_for((uint64_t)E - 1);
  p.bbits = bits_for(nb - 1);
  const int bits = p.ebits + p.bbits;
  if (bits > 64) return false;
  p.passes = (bits + kMaxDigitBits - 1) / kMaxDigitBits;
  if (p.passes < 1) p.passes = 1;
  for (int i = 0, at = 0; i < p.passes; ++i) {  // spread the key bits evenly over the passes
    const int w = (bits - at + (p.passes - i) - 1) / (p.passes - i);
    p.shift[i] = at;
    p.width[i] = w < 1 ? 1 : w;
    at += w;
  }
  p.tile = kSortTile;
  p.sort_blocks = (uint32_t)((p.N + kSortTile - 1) / kSortTile);
  p.seg_blocks = (uint32_t)((p.N + kSegTile - 1) / kSegTile);
  p.fused = p.sort_blocks <= (uint32_t)kFusedMaxTiles;
  p.msd = p.fused && p.N > kSmallMaxN && bits > kMaxDigitBits;
  if (p.msd && p.N < 131072) {  // small inputs: smaller tiles put more workgroups on the one global pass
    p.tile = p.N <= 32768 ? 512 : 1024;
    p.sort_blocks = (uint32_t)((p.N + p.tile - 1) / p.tile);
  }
  if (p.msd) {
    p.top_width = kMaxDigitBits;
    p.top_shift = bits - kMaxDigitBits;
    const int rem = p.top_shift;
    const int lp = (rem + kMaxDigitBits - 1) / kMaxDigitBits;
    p.low_passes = lp;
    for (int i = 0, at = 0; i < lp; ++i) {
      const int w = (rem - at + (lp - i) - 1) / (lp - i);
      p.low_shift[i] = at;
      p.low_width[i] = w;
      at += w;
    }
  }
  size_t off = 0;
  for (int i = 0; i < 2; ++i) {
    p.off_key[i] = off;
    off = align256(off + (size_t)p.N * 8);
  }
  for (int i = 0; i < 2; ++i) {
    p.off_idx[i] = off;
    off = align256(off + (size_t)p.N * 4);
  }
  p.off_table = off;
  off = align256(off + (size_t)kGroupBins * p.sort_blocks * 4);
  p.off_blocksum = off;
  off = align256(off + ((size_t)p.seg_blocks + 1) * 4);
  p.off_binstart = off;
  off = align256(off + ((size_t)kGroupBins + 3) * 4);
  p.off_chunktbl = off;
  const size_t max_chunks = (size_t)kGroupBins + (size_t)((p.N + kBinChunk - 1) / kBinChunk);  // one per non-empty bin and per kBinChunk keys
  off = align256(off + max_chunks * 4);
  p.off_chunkheads = off;
  off = align256(off + max_chunks * 16);
  const size_t windows = 2 * (size_t)((p.N + kCentroidWindow - 1) / kCentroidWindow);
  p.off_partial = off;
  off = align256(off + windows * (size_t)d * 4);
  p.off_counters = off;
  // every numbering tile clears the counters of its whole tile, so the count is rounded up to whole tiles
  off = align256(off + (size_t)p.seg_blocks * (2 * kSegTile / kCentroidWindow) * 4);
  p.total_bytes = off;
  *plan = p;
  return true;
}

// A launch followed by a look at its status: a refused launch ends the call before anything else is enqueued.
#define LSHMOE_LAUNCH(...)                                                        \
  do {                                                                            \
    hipLaunchKernelGGL(__VA_ARGS__);                                              \
    if (hipError_t launch_err = hipGetLastError(); launch_err != hipSuccess) return launch_err; \
  } while (0)

hipError_t launch_group(const GroupPlan& plan, const int32_t* expert, const uint64_t* bucket, int k, int E,
                        int32_t* seg_offsets, int32_t* seg_expert, int32_t* expert_offsets, int32_t* perm,
                        int32_t* seg_of, int32_t* num_segments, char* ws, hipStream_t stream) {
  const uint32_t N = (uint32_t)plan.N;
  uint64_t* keybuf[2] = {(uint64_t*)(ws + plan.off_key[0]), (uint64_t*)(ws + plan.off_key[1])};
  int32_t* idxbuf[2] = {(int32_t*)(ws + plan.off_idx[0]), (int32_t*)(ws + plan.off_idx[1])};
  uint32_t* table = (uint32_t*)(ws + plan.off_table);
  uint32_t* blocksum = (uint32_t*)(ws + plan.off_blocksum);
  const uint32_t nblk = plan.sort_blocks;
  const dim3 grid(nblk), block(kSortThreads);

  KeySource src{expert, bucket, nullptr, nullptr, (uint32_t)k, (uint32_t)E, plan.bbits};
  if (plan.N <= kSmallMaxN) {
    SmallArgs a{};
    a.passes = plan.passes;
    a.bbits = plan.bbits;
    for (int p = 0; p < plan.passes; ++p) {
      a.shift[p] = plan.shift[p];
      a.width[p] = plan.width[p];
    }
    a.N = N;
    a.E = (uint32_t)E;
    a.keybuf[0] = keybuf[0]; a.keybuf[1] = keybuf[1];
    a.idxbuf[0] = idxbuf[0]; a.idxbuf[1] = idxbuf[1];
    a.seg_offsets = seg_offsets; a.seg_expert = seg_expert; a.expert_offsets = expert_offsets;
    a.perm = perm; a.seg_of = seg_of; a.num_segments = num_segments;
    a.window_counters = (uint32_t*)(ws + plan.off_counters);
    LSHMOE_LAUNCH(small_group_kernel, dim3(1), dim3(kSmallWaves * 64), 0, stream, src, a);
    return hipGetLastError();
  }
  const uint64_t* sorted_key = nullptr;
  if (plan.msd) {
    uint32_t* bin_start = (uint32_t*)(ws + plan.off_binstart);
    PassArgs a{};
    a.shift = plan.top_shift;
    a.mask = (1u << plan.top_width) - 1u;
    a.nblk = nblk;
    a.table = table;
    a.bin_start = bin_start;
    a.chunk_tbl = (uint32_t*)(ws + plan.off_chunktbl);
    // the histogram kernel also clears the per-tile head counts that the bin kernels add to
    hipError_t e = hipSuccess;
#define LSHMOE_GLOBAL_PASS(TILE)                                                                                     \
    LSHMOE_LAUNCH((sort_hist_kernel<true, true, TILE>), grid, block, 0, stream, src, N, a.shift, a.mask, nblk, table, \
                  blocksum, plan.seg_blocks + 1);                                                                       \
    e = launch_scatter<true, true, TILE>(src, N, a, keybuf[0], idxbuf[0], stream)
    if (plan.tile == 512) { LSHMOE_GLOBAL_PASS(512); }
    else if (plan.tile == 1024) { LSHMOE_GLOBAL_PASS(1024); }
    else { LSHMOE_GLOBAL_PASS(kSortTile); }
#undef LSHMOE_GLOBAL_PASS
    if (e != hipSuccess) return e;
    BinSortArgs b{};
    b.bin_start = bin_start;
    b.chunk_tbl = a.chunk_tbl;
    b.key[0] = keybuf[0]; b.key[1] = keybuf[1];
    b.idx[0] = idxbuf[0];
    b.perm = perm;
    b.passes = plan.low_passes;
    for (int p = 0; p < plan.low_passes; ++p) {
      b.shift[p] = plan.low_shift[p];
      b.width[p] = plan.low_width[p];
    }
    const int sub_bits = plan.top_shift < 8 ? plan.top_shift : 8;
    b.sub_shift = plan.top_shift - sub_bits;
    b.sub_mask = (1u << sub_bits) - 1u;
    b.tile_heads = blocksum;
    b.chunk_heads = (uint4*)(ws + plan.off_chunkheads);
    const dim3 chunks((uint32_t)kGroupBins + (N + kBinChunk - 1) / kBinChunk), threads(kBinThreads);
    LSHMOE_LAUNCH(bin_sort_kernel, chunks, threads, kBinSortLds, stream, b);
    LSHMOE_LAUNCH(bin_merge_kernel, dim3(chunks.x * kMergeSlices < 512u ? chunks.x * kMergeSlices : 512u), threads, 0, stream, b);
    // the heads per numbering tile are known: number the clusters (the tile count is within kSelfPrefixMaxTiles here)
    LSHMOE_LAUNCH(seg_write_kernel<true>, dim3(plan.seg_blocks), dim3(kSegThreads), 0, stream,
                       (const uint64_t*)keybuf[1], perm, N, (uint32_t)E, plan.bbits, blocksum, seg_offsets, seg_expert,
                       expert_offsets, seg_of, num_segments, (uint32_t*)(ws + plan.off_counters),
                       (const uint4*)b.chunk_heads, (const uint32_t*)(bin_start + kGroupBins + 1));
    return hipGetLastError();
  }
  for (int p = 0; p < (plan.msd ? 0 : plan.passes); ++p) {
    const bool last = p == plan.passes - 1;
    uint64_t* dkey = keybuf[p & 1];
    int32_t* didx = last ? perm : idxbuf[p & 1];
    PassArgs a{};
    a.shift = plan.shift[p];
    a.mask = (1u << plan.width[p]) - 1u;
    a.nblk = nblk;
    a.table = table;
    hipError_t e = hipSuccess;
    if (plan.fused) {
      if (p == 0) {
        LSHMOE_LAUNCH((sort_hist_kernel<true, true>), grid, block, 0, stream, src, N, a.shift, a.mask, nblk, table);
        e = launch_scatter<true, true>(src, N, a, dkey, didx, stream);
      } else {
        LSHMOE_LAUNCH((sort_hist_kernel<false, true>), grid, block, 0, stream, src, N, a.shift, a.mask, nblk, table);
        e = launch_scatter<false, true>(src, N, a, dkey, didx, stream);
      }
    } else {
      if (p == 0)
        LSHMOE_LAUNCH((sort_hist_kernel<true, false>), grid, block, 0, stream, src, N, a.shift, a.mask, nblk, table);
      else
        LSHMOE_LAUNCH((sort_hist_kernel<false, false>), grid, block, 0, stream, src, N, a.shift, a.mask, nblk, table);
      LSHMOE_LAUNCH(scan_kernel, dim3(1), dim3(1024), 0, stream, table, (a.mask + 1u) * nblk);
      e = p == 0 ? launch_scatter<true, false>(src, N, a, dkey, didx, stream)
                 : launch_scatter<false, false>(src, N, a, dkey, didx, stream);
    }
    if (e != hipSuccess) return e;
    src.key = dkey;
    src.idx = didx;
    sorted_key = dkey;
  }
  const uint32_t sblk = plan.seg_blocks;
  LSHMOE_LAUNCH(seg_count_kernel, dim3(sblk), dim3(kSegThreads), 0, stream, sorted_key, N, sblk, blocksum,
                     (uint32_t*)(ws + plan.off_counters));
  if (sblk <= (uint32_t)kSelfPrefixMaxTiles) {
    LSHMOE_LAUNCH(seg_write_kernel<true>, dim3(sblk), dim3(kSegThreads), 0, stream, sorted_key, perm, N,
                       (uint32_t)E, plan.bbits, blocksum, seg_offsets, seg_expert, expert_offsets, seg_of,
                       num_segments);
  } else {
    LSHMOE_LAUNCH(scan_kernel, dim3(1), dim3(1024), 0, stream, blocksum, sblk + 1);
    LSHMOE_LAUNCH(seg_write_kernel<false>, dim3(sblk), dim3(kSegThreads), 0, stream, sorted_key, perm, N,
                       (uint32_t)E, plan.bbits, blocksum, seg_offsets, seg_expert, expert_offsets, seg_of,
                       num_segments);
  }
  return hipGetLastError();
}

#undef LSHMOE_LAUNCH

}  // namespace lshmoe
