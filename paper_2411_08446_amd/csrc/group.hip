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
//    bin on the remaining bits inside LDS (in chunks of 2048 keys; the chunks of
//    a bin that has several are merged in the same launch by the workgroups
//    that sorted them, the later of two neighbours each time), and one launch
//    that numbers the clusters from the head counts the bin kernel left per
//    tile: four launches whatever the key width.  (Before: a histogram and a
//    scatter launch per 9 key bits, and a counting launch.)
//  - larger: least-significant-digit radix passes of histogram,
//    single-workgroup scan of the (bin, tile) table and scatter.
//
// Ranks inside a tile of 2048 keys come from wave ballots: a wave of 64 keys
// finds, for every lane, the lanes holding the same digit; tile order equals
// element order, which keeps the sort stable.  (Accumulating the next pass's
// table with global atomics from inside the scatter was measured slower than
// the separate histogram launch: device-scope atomics cost ~8 us per pass.)
#include <atomic>
#include <cstddef>

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
  if (threadIdx.x == 0) bin_start[kGroupBins + 1] = half + rest;
}

struct PassArgs {
  int shift;            // this pass's digit is (key >> shift) & mask
  uint32_t mask;
  uint32_t nblk;
  const uint32_t* table;  // FUSED: tile-major counts of this pass; else the scanned bin-major offsets
  uint32_t* bin_start;    // FUSED, optional: block 0 writes the first output position of every bin, then N,
  uint32_t* chunk_tbl;    // then the number of chunks; and the chunk table
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
// key bits inside LDS; the chunks of a bin of several are then merged pairwise, in the same launch (merge_up).
// That replaces a histogram and a scatter launch per further digit by one launch.
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
  const uint32_t* bin_start;  // [bins + 1], then [bins + 1] = number of chunks
  const uint32_t* chunk_tbl;  // chunk w is chunk (entry & 0xffff) of bin (entry >> 16)
  uint64_t* key[2];           // [0]: keys after the global pass; [1]: receives the sorted keys
  int32_t* idx[2];            // [0]: assignment ids after the global pass; [1]: second buffer of the chunk merges
  int32_t* perm;              // receives the sorted assignment ids
  int passes;                 // radix passes over the low key bits
  int shift[8], width[8];     // their digits, least significant first
  int sub_shift;              // sub-bin of a key is (key >> sub_shift) & sub_mask
  uint32_t sub_mask;
  uint32_t* tile_heads;       // [tiles of kSegTile positions]: cluster heads per tile of bins of several chunks (atomics)
  uint4* chunk_heads;         // [chunks]: {first tile, heads in it, in the next, in the one after} of a bin of one chunk
  uint32_t* merge_arrivals;   // [chunks], zero on entry: runs that have arrived at a merge, indexed by the chunk that
                              // starts the merge's right-hand run
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

// Merge of the sorted chunks of a bin that has several, inside the launch that sorts the chunks.  The chunks of
// the bin are the leaves of a binary tree: the node of level j that covers chunks [i 2^j, (i + 1) 2^j) merges the
// sorted runs of its two children.  Nobody waits: a workgroup that has finished a run adds one to the node's
// arrival counter; the first to arrive leaves, the second finds both runs complete (fence, device-scope atomic,
// fence), merges them and carries the result one level up.  A run without a right-hand neighbour is copied, so
// that every run of a level sits in the same one of the two buffers and a merge never writes where it reads; the
// chunk sort starts in the buffer from which the root's output lands in the final arrays.  The merge is stable
// (on equal keys the left run, i.e. the lower assignment ids, goes first) and proceeds in tiles of kBinChunk
// outputs: the tile's share of either run is found by a search along the merge path (all boundaries at once, one
// per thread), staged in LDS, merged there (every thread a run of consecutive outputs) and written out in order.
// The root also counts the cluster heads per numbering tile.  Depth is log2 of the bin's chunk count; a node is one
// workgroup, so bins of several chunks take about twice as long as with the separate merge launch this replaces
// (four workgroups per chunk) - which every other input paid for with an idle launch.
struct MergeLds {
  uint64_t in_key[kBinChunk];    // the tile's share of the left run, then of the right run
  uint64_t out_key[kBinChunk];
  int32_t in_idx[kBinChunk];
  int32_t out_idx[kBinChunk];
};
static_assert(sizeof(MergeLds) == 2 * (size_t)kBinChunk * (8 + 4), "the merge reuses the chunk sort's dynamic LDS");
struct MergeState {                    // small LDS state of a merge, double buffered by tile parity
  uint32_t tile_cnt[2][kChunkTiles];   // heads of a tile's outputs per numbering tile
  uint64_t last_key[2];                // a tile's last output
  uint32_t flag;                       // what the arrival counter held
};

// Number of elements of the left run among the first `diag` outputs of the stable merge of A[0, na) and B[0, nb):
// the first x in [lo, hi] for which "A[x] goes before B[diag - 1 - x]" no longer holds.  Sixteen probes per step
// instead of one: the runs were written by other compute units and every probe is a trip to memory, so the
// number of dependent steps is what counts (4 for 65536 keys instead of 16).
__device__ __forceinline__ uint32_t merge_path_split(const uint64_t* A, uint32_t na, const uint64_t* B, uint32_t nb,
                                                     uint32_t diag) {
  constexpr int kProbes = 16;
  uint32_t lo = diag > nb ? diag - nb : 0u, hi = min(diag, na);
  while (lo < hi) {
    const uint32_t w = (hi - lo + kProbes - 1) / kProbes;   // >= 1
    uint64_t av[kProbes], bv[kProbes];
#pragma unroll
    for (int i = 0; i < kProbes; ++i) {                      // probe i sits at lo + i w; past hi it re-reads the last valid one
      const uint32_t x = min(lo + (uint32_t)i * w, hi - 1);  // lo <= x < hi <= min(diag, na); diag - 1 - x in [0, nb)
      av[i] = A[x];
      bv[i] = B[diag - 1 - x];
    }
    uint32_t before = 0;                                     // probes whose A element goes first: a prefix of them
#pragma unroll
    for (int i = 0; i < kProbes; ++i) before += (lo + (uint32_t)i * w < hi && av[i] <= bv[i]) ? 1u : 0u;
    if (before == 0) return lo;
    const uint32_t next = lo + before * w;                   // the first probe that failed, if there is one below hi
    lo = lo + (before - 1) * w + 1;
    hi = before < (uint32_t)kProbes && next < hi ? next : hi;
  }
  return lo;
}

// Slot of element i of a staged tile.  The bisection below probes indices that differ by multiples of a power of
// two; stored plainly those all fall into the same LDS bank (up to 64 lanes one after the other); swapping the low
// five index bits around by the next ten spreads them.
__device__ __forceinline__ uint32_t merge_slot(uint32_t i) { return i ^ ((i >> 5) & 31u) ^ ((i >> 10) & 31u); }
static_assert(kBinChunk <= (1 << 15), "merge_slot permutes indices below 2^15 inside blocks of 32");

// Barrier that orders LDS accesses only: unlike __syncthreads() it does not wait for the wave's global loads and
// stores, which inside the merge loop are a prefetch that should stay in flight and outputs nobody in the workgroup
// reads before the merge ends.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Every thread of the workgroup calls it (kBinThreads threads).  src/dst: the two buffers; the runs are
// src[lo_a, lo_a + na) and src[lo_a + na, lo_a + na + nb); the output is dst[lo_a, lo_a + na + nb).
// count_heads: also adds the heads of the output to tile_heads (the output is final).
// (No __restrict__ on the runs: other workgroups wrote them during this launch, and every load of them has to stay
// an ordinary vector load behind the fence.)
__device__ __forceinline__ void merge_runs(const uint64_t* src_key, const int32_t* src_idx, uint64_t* dst_key, int32_t* dst_idx,
                           uint32_t lo_a, uint32_t na, uint32_t nb, bool count_heads, uint32_t* tile_heads, MergeLds& m,
                           uint32_t* split /*[kFusedMaxTiles + 1] in LDS*/, MergeState& st) {
  constexpr int kItems = kBinChunk / kBinThreads;   // elements of a tile per thread: 8
  const uint64_t* A = src_key + lo_a;
  const uint64_t* B = A + na;
  const uint32_t n = na + nb, tiles = (n + kBinChunk - 1) / kBinChunk;   // tiles <= kFusedMaxTiles
  __syncthreads();   // LDS of an earlier merge (or of the chunk sort) is no longer read
  for (uint32_t t = threadIdx.x; t <= tiles; t += kBinThreads)
    split[t] = t == 0 ? 0u : t == tiles ? na : merge_path_split(A, na, B, nb, t * kBinChunk);
  __syncthreads();
  // a tile's inputs are fetched into registers one tile ahead, so that the loads fly while the tile before is ranked
  uint64_t pk[kItems];
  int32_t pi[kItems];
  auto fetch = [&](uint32_t t) {
    const uint32_t a0 = split[t], a1 = split[t + 1];
    const uint32_t out0 = t * kBinChunk;
    const uint32_t b0 = out0 - a0, ca = a1 - a0;
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
      const uint32_t e = threadIdx.x + q * kBinThreads;   // past the tile's last element: clamped, never used
      const uint32_t from = min(e < ca ? lo_a + a0 + e : lo_a + na + b0 + (e - ca), lo_a + n - 1);
      pk[q] = src_key[from];
      pi[q] = src_idx[from];
    }
  };
  fetch(0);
  for (uint32_t t = 0; t < tiles; ++t) {
    const uint32_t a0 = split[t], a1 = split[t + 1];
    const uint32_t out0 = t * kBinChunk, out1 = min(out0 + (uint32_t)kBinChunk, n);
    const uint32_t ca = a1 - a0, cn = out1 - out0, cb = cn - ca;   // cn <= kBinChunk
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
      const uint32_t e = threadIdx.x + q * kBinThreads;
      if (e < cn) {
        m.in_key[merge_slot(e)] = pk[q];
        m.in_idx[e] = pi[q];
      }
    }
    if (count_heads && threadIdx.x < (uint32_t)kChunkTiles) st.tile_cnt[t & 1][threadIdx.x] = 0;
    lds_barrier();
    if (t + 1 < tiles) fetch(t + 1);
    if (count_heads && t > 0 && threadIdx.x < (uint32_t)kChunkTiles && st.tile_cnt[(t - 1) & 1][threadIdx.x] != 0)
      atomicAdd(&tile_heads[((lo_a + out0 - kBinChunk) >> kSegTileBits) + threadIdx.x], st.tile_cnt[(t - 1) & 1][threadIdx.x]);
    {
      // Every thread produces kItems consecutive outputs of the tile: one search along the merge path finds how
      // many of the outputs before its first one come from the left part, then it merges step by step (on equal
      // keys the left part goes first).  A wave runs alone on its SIMD here, so instructions per key are what
      // counts: ranking every key by a bisection of its own took eight times as many.
      const uint32_t diag = min(threadIdx.x * (uint32_t)kItems, cn);
      // (plain bisection: in LDS a probe is cheap and the sixteen-way search's extra instructions cost more)
      uint32_t lo = diag > cb ? diag - cb : 0u, hi = min(diag, ca);
      while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;   // mid < ca; diag - 1 - mid in [0, cb)
        if (m.in_key[merge_slot(mid)] <= m.in_key[merge_slot(ca + diag - 1 - mid)]) lo = mid + 1; else hi = mid;
      }
      uint32_t ai = lo, bi = ca + (diag - lo);   // next element of either part, as indices into in_key
      const uint32_t last = kBinChunk - 1;     // reads past a part's end are clamped and never chosen
      uint64_t ka = m.in_key[merge_slot(min(ai, last))], kb = m.in_key[merge_slot(min(bi, last))];
#pragma unroll
      for (int q = 0; q < kItems; ++q) {
        const uint32_t at = diag + q;
        const bool take_a = ai < ca && (bi >= cn || ka <= kb);
        if (at < cn) {
          m.out_key[at] = take_a ? ka : kb;
          m.out_idx[at] = m.in_idx[take_a ? ai : bi];
        }
        if (take_a) { ++ai; ka = m.in_key[merge_slot(min(ai, last))]; }
        else { ++bi; kb = m.in_key[merge_slot(min(bi, last))]; }
      }
    }
    lds_barrier();
    const uint32_t first_tile = (lo_a + out0) >> kSegTileBits;
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
      const uint32_t e = threadIdx.x + q * kBinThreads;
      if (e < cn) {
        const uint64_t key = m.out_key[e];
        dst_key[lo_a + out0 + e] = key;
        dst_idx[lo_a + out0 + e] = m.out_idx[e];
        if (e == cn - 1) st.last_key[t & 1] = key;   // the key before the next tile's first output
        if (count_heads) {
          // the first key of a bin always starts a cluster: the key before it belongs to another bin
          const bool head = e == 0 ? (t == 0 || st.last_key[(t - 1) & 1] != key) : m.out_key[e - 1] != key;
          if (head) atomicAdd(&st.tile_cnt[t & 1][((lo_a + out0 + e) >> kSegTileBits) - first_tile], 1u);
        }
      }
    }
    // the next tile's staging writes touch in_*, which nobody reads any more; out_* is read until the barrier that
    // follows those writes, and written again only after it
  }
  __syncthreads();
  if (count_heads && threadIdx.x < (uint32_t)kChunkTiles && st.tile_cnt[(tiles - 1) & 1][threadIdx.x] != 0)
    atomicAdd(&tile_heads[((lo_a + (tiles - 1) * kBinChunk) >> kSegTileBits) + threadIdx.x], st.tile_cnt[(tiles - 1) & 1][threadIdx.x]);
}

// The first level of the tree merges two chunks: at most 2 kBinChunk keys, which fit in the merge's LDS block at once
// (its input and output halves side by side).  No tile boundaries to search in memory, one trip for the inputs, and
// every thread merges 2 kBinChunk / kBinThreads consecutive outputs: half the time of merge_runs on the same pair,
// and bins of two chunks are the commonest case of a bin of several.  Same arguments as merge_runs.
__device__ __forceinline__ void merge_pair(const uint64_t* src_key, const int32_t* src_idx, uint64_t* dst_key, int32_t* dst_idx,
                                           uint32_t lo_a, uint32_t na, uint32_t nb, bool count_heads, uint32_t* tile_heads,
                                           MergeLds& m, MergeState& st) {
  constexpr int kItems = 2 * kBinChunk / kBinThreads;   // 16
  constexpr uint32_t kLast = 2 * kBinChunk - 1;
  static_assert(offsetof(MergeLds, out_key) == sizeof(uint64_t) * kBinChunk &&
                    offsetof(MergeLds, out_idx) == offsetof(MergeLds, in_idx) + sizeof(int32_t) * kBinChunk,
                "the two halves of the key and of the id arrays are adjacent");
  uint64_t* K = m.in_key;   // [2 kBinChunk]
  int32_t* I = m.in_idx;    // [2 kBinChunk]
  uint32_t* heads = &st.tile_cnt[0][0];   // 2 kBinChunk positions touch at most 2 kBinChunk / kSegTile + 1 numbering tiles
  static_assert(2 * kBinChunk / kSegTile + 1 <= 2 * kChunkTiles, "head counters of a pair fit the merge state");
  const uint32_t n = na + nb;   // <= 2 kBinChunk
  __syncthreads();   // LDS of the chunk sort is no longer read
  {
    uint64_t pk[kItems];
    int32_t pi[kItems];
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
      const uint32_t e = min(threadIdx.x + q * kBinThreads, n - 1);
      pk[q] = src_key[lo_a + e];
      pi[q] = src_idx[lo_a + e];
    }
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
      const uint32_t e = threadIdx.x + q * kBinThreads;
      if (e < n) {
        K[merge_slot(e)] = pk[q];
        I[e] = pi[q];
      }
    }
  }
  if (threadIdx.x < 2u * kChunkTiles) heads[threadIdx.x] = 0;
  lds_barrier();
  uint64_t ok[kItems];
  int32_t oi[kItems];
  const uint32_t diag = min(threadIdx.x * (uint32_t)kItems, n);
  {
    uint32_t lo = diag > nb ? diag - nb : 0u, hi = min(diag, na);
    while (lo < hi) {
      const uint32_t mid = (lo + hi) >> 1;   // mid < na; diag - 1 - mid in [0, nb)
      if (K[merge_slot(mid)] <= K[merge_slot(na + diag - 1 - mid)]) lo = mid + 1; else hi = mid;
    }
    uint32_t ai = lo, bi = na + (diag - lo);   // next element of either run, as indices into K
    uint64_t ka = K[merge_slot(min(ai, kLast))], kb = K[merge_slot(min(bi, kLast))];
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
      const bool take_a = ai < na && (bi >= n || ka <= kb);
      ok[q] = take_a ? ka : kb;
      oi[q] = I[min(take_a ? ai : bi, kLast)];
      if (take_a) { ++ai; ka = K[merge_slot(min(ai, kLast))]; }
      else { ++bi; kb = K[merge_slot(min(bi, kLast))]; }
    }
  }
  lds_barrier();   // every thread has read its inputs: the block now takes the outputs, in order
#pragma unroll
  for (int q = 0; q < kItems; ++q) {
    const uint32_t at = diag + q;
    if (at < n) {
      K[at] = ok[q];
      I[at] = oi[q];
    }
  }
  lds_barrier();
  const uint32_t first_tile = lo_a >> kSegTileBits;
#pragma unroll
  for (int q = 0; q < kItems; ++q) {
    const uint32_t e = threadIdx.x + q * kBinThreads;
    if (e < n) {
      const uint64_t key = K[e];
      dst_key[lo_a + e] = key;
      dst_idx[lo_a + e] = I[e];
      // counted only at the root, whose first key is the bin's first and always starts a cluster
      if (count_heads && (e == 0 || K[e - 1] != key)) atomicAdd(&heads[((lo_a + e) >> kSegTileBits) - first_tile], 1u);
    }
  }
  __syncthreads();
  if (count_heads && threadIdx.x < 2u * kChunkTiles && heads[threadIdx.x] != 0)
    atomicAdd(&tile_heads[first_tile + threadIdx.x], heads[threadIdx.x]);
}

// Called by every thread of a workgroup that has just written chunk `chunk` of a bin of several chunks, sorted,
// into buffer `start_buf`.  Returns when the workgroup has nothing left to merge.
__device__ __forceinline__ void merge_up(const BinSortArgs& a, uint32_t lo_bin, uint32_t hi_bin, uint32_t chunk, uint32_t first_chunk_slot,
                         MergeLds& m, uint32_t* split, MergeState& st) {
  const uint32_t chunks = (hi_bin - lo_bin + kBinChunk - 1) / kBinChunk;
  int levels = 0;
  while ((1u << levels) < chunks) ++levels;
  uint32_t buf = (levels & 1) ? 0u : 1u;          // where the sorted chunks are: the root's output lands in buffer 1
  for (int j = 1; j <= levels; ++j, buf ^= 1u) {
    const uint32_t left0 = (chunk >> j) << j, right0 = left0 + (1u << (j - 1));
    const uint32_t lo_a = lo_bin + left0 * kBinChunk;
    const bool final_level = j == levels;
    const uint64_t* src_key = buf ? a.key[1] : a.key[0];
    const int32_t* src_idx = buf ? a.idx[1] : a.idx[0];
    uint64_t* dst_key = buf ? a.key[0] : a.key[1];
    int32_t* dst_idx = final_level ? a.perm : buf ? a.idx[0] : a.idx[1];   // the root writes buffer 1's keys and the result ids
    if (right0 >= chunks) {
      // no right-hand run (never at the root): move the run to the buffer its level's outputs live in
      const uint32_t n = hi_bin - lo_a;
      for (uint32_t e = threadIdx.x; e < n; e += kBinThreads) {
        dst_key[lo_a + e] = src_key[lo_a + e];
        dst_idx[lo_a + e] = src_idx[lo_a + e];
      }
      __syncthreads();   // the next level may copy again, reading what other threads wrote here
      continue;
    }
    __threadfence();      // this workgroup's run is visible device-wide before the counter moves
    __syncthreads();
    if (threadIdx.x == 0) st.flag = atomicAdd(&a.merge_arrivals[first_chunk_slot + right0], 1u);
    __syncthreads();
    if (st.flag == 0u) return;   // the other run is still being made: its workgroup will find this one complete
    __threadfence();      // second to arrive: the other run is complete and visible
    const uint32_t na = (right0 - left0) * kBinChunk;             // a left-hand run is always full
    const uint32_t end = min(lo_bin + (left0 + (1u << j)) * kBinChunk, hi_bin);
    if (j == 1)
      merge_pair(src_key, src_idx, dst_key, dst_idx, lo_a, na, end - lo_a - na, final_level, a.tile_heads, m, st);
    else
      merge_runs(src_key, src_idx, dst_key, dst_idx, lo_a, na, end - lo_a - na, final_level, a.tile_heads, m, split, st);
  }
}

__global__ __launch_bounds__(kBinThreads) void bin_sort_kernel(BinSortArgs a) {
  extern __shared__ uint64_t bin_lds[];            // radix way: keys [2][kBinChunk], then ids [2][kBinChunk]
  __shared__ uint32_t cnt[kBinWaves][kGroupBins];  // 8 KB; the sub-bin way keeps its keys here
  __shared__ uint32_t place_s[kBinFast];           // sub-bin way: a key's place in the chunk before sorting
  __shared__ uint32_t sub_cnt[kSubBins], sub_base[kSubBins];
  __shared__ uint32_t wave_sum[kBinWaves];
  __shared__ uint32_t tile_cnt[kChunkTiles];
  __shared__ MergeState merge_state;
  static_assert(sizeof(cnt) >= (kFusedMaxTiles + 1) * sizeof(uint32_t), "the merge keeps its tile boundaries in cnt");
  if (blockIdx.x >= a.bin_start[kGroupBins + 1]) return;
  if (threadIdx.x < (uint32_t)kChunkTiles) tile_cnt[threadIdx.x] = 0;  // a barrier follows on every way
  const uint32_t entry = a.chunk_tbl[blockIdx.x];
  const uint32_t bin = entry >> 16, chunk = entry & 0xffffu;
  const uint32_t lo_bin = a.bin_start[bin], hi_bin = a.bin_start[bin + 1];
  const uint32_t lo = lo_bin + chunk * kBinChunk, hi = min(lo + (uint32_t)kBinChunk, hi_bin);
  const uint32_t n = hi - lo;
  // a bin of one chunk is finished here; the chunks of a larger bin are merged by the workgroups that sorted
  // them (merge_up), starting from the buffer that makes the last merge land in the final arrays
  const bool alone = hi_bin - lo_bin <= (uint32_t)kBinChunk;
  uint32_t start_buf = 0;
  if (!alone) {
    const uint32_t chunks = (hi_bin - lo_bin + kBinChunk - 1) / kBinChunk;
    int levels = 0;
    while ((1u << levels) < chunks) ++levels;
    start_buf = (levels & 1) ? 0u : 1u;
  }
  uint64_t* out_key = alone || start_buf ? a.key[1] : a.key[0];
  int32_t* out_idx = alone ? a.perm : start_buf ? a.idx[1] : a.idx[0];
  MergeLds& merge_lds = *reinterpret_cast<MergeLds*>(bin_lds);
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
      if (!alone) merge_up(a, lo_bin, hi_bin, chunk, blockIdx.x - chunk, merge_lds, &cnt[0][0], merge_state);
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
  if (!alone) merge_up(a, lo_bin, hi_bin, chunk, blockIdx.x - chunk, merge_lds, &cnt[0][0], merge_state);
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
  const size_t max_chunks = (size_t)kGroupBins + (size_t)((p.N + kBinChunk - 1) / kBinChunk);  // one per non-empty bin and per kBinChunk keys
  p.off_blocksum = off;   // head counts per numbering tile (+ 1), then the merge arrival counters: cleared together
  off = align256(off + ((size_t)p.seg_blocks + 1 + max_chunks) * 4);
  p.off_binstart = off;
  off = align256(off + ((size_t)kGroupBins + 2) * 4);
  p.off_chunktbl = off;
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
    // the histogram kernel also clears the per-tile head counts and the arrival counters that the bin kernel adds to
    const uint32_t max_chunks = (uint32_t)kGroupBins + (N + kBinChunk - 1) / kBinChunk;
    hipError_t e = hipSuccess;
#define LSHMOE_GLOBAL_PASS(TILE)                                                                                     \
    LSHMOE_LAUNCH((sort_hist_kernel<true, true, TILE>), grid, block, 0, stream, src, N, a.shift, a.mask, nblk, table, \
                  blocksum, plan.seg_blocks + 1 + max_chunks);                                                          \
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
    b.idx[0] = idxbuf[0]; b.idx[1] = idxbuf[1];
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
    b.merge_arrivals = blocksum + plan.seg_blocks + 1;
    const dim3 chunks(max_chunks), threads(kBinThreads);
    LSHMOE_LAUNCH(bin_sort_kernel, chunks, threads, kBinSortLds, stream, b);
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
