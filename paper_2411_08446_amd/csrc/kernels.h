// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "common.h"

namespace lshmoe {

// ---- step 1: hash -------------------------------------------------------
hipError_t launch_hash(const void* tokens, const void* rot, int64_t T, int d, int L, int r, bool bf16,
                       uint64_t* bucket, hipStream_t stream);

// Hash plus E rows of a gate projection in one pass over the tokens (logits[T][E], binary32).  Supported shapes:
// hash_gate_supported (r a multiple of 8, rows of whole 512-byte blocks, E <= 128).
bool hash_gate_supported(int d, int r, int E, bool bf16);
hipError_t launch_hash_gate(const void* tokens, const void* rot, const void* gate_w, int64_t T, int d, int L, int r, int E,
                            bool bf16, uint64_t* bucket, float* logits, hipStream_t stream);

// Spherical hash (one bit per sphere, B <= 63 spheres): bucket[t] = B-bit code, bit 0 most significant.
hipError_t launch_hash_sphere(const void* tokens, const void* pivots, const float* radius_sq, int64_t T, int d, int B,
                              bool bf16, uint64_t* bucket, hipStream_t stream);

// ---- step 2: group ------------------------------------------------------
constexpr int kSortTile = 2048;            // assignments per sort tile
constexpr int kSegTile = 1024;             // sorted positions per cluster-numbering tile
constexpr int kMaxDigitBits = 9;           // radix digit width limit
constexpr int kGroupBins = 1 << kMaxDigitBits;
constexpr int kFusedMaxTiles = 256;        // up to this many sort tiles: no scan launch
constexpr int kSelfPrefixMaxTiles = 4096;  // up to this many numbering tiles: no scan launch
constexpr int kSmallMaxN = 4096;           // up to this many assignments: one workgroup, one launch

struct GroupPlan {
  int64_t N;
  int ebits, bbits;      // key = expert << bbits | bucket
  int passes;            // radix passes over ebits + bbits key bits
  int shift[8], width[8];  // digit of pass p is (key >> shift[p]) & ((1 << width[p]) - 1)
  bool fused;            // scatter blocks derive their offsets themselves (small inputs)
  bool msd;              // one global pass on the top digit, then every bin sorted by one workgroup
  int top_shift, top_width;        // msd: the global pass's digit
  int low_passes;                  // msd: radix passes over the remaining bits
  int low_shift[8], low_width[8];
  int tile;              // assignments per sort tile (kSortTile, or less on small inputs)
  uint32_t sort_blocks;  // sort tiles
  uint32_t seg_blocks;   // tiles of kSegTile sorted positions
  // byte offsets into the workspace
  size_t off_key[2], off_idx[2], off_table, off_blocksum, off_binstart, off_chunktbl, off_chunkheads;
  size_t off_partial, off_counters;  // window sums and window counters of the centroid step
  size_t total_bytes;
};

constexpr int kCentroidWindow = 128;  // clusters with more members are summed in windows of this many positions

// Fills the plan (d = elements per token row); returns false when ebits + bbits > 64.
bool plan_group(int64_t T, int d, int k, int E, int L, int r, GroupPlan* plan);

hipError_t launch_group(const GroupPlan& plan, const int32_t* expert, const uint64_t* bucket, int k, int E,
                        int32_t* seg_offsets, int32_t* seg_expert, int32_t* expert_offsets, int32_t* perm,
                        int32_t* seg_of, int32_t* num_segments, char* workspace, hipStream_t stream);

// ---- step 3: centroid ---------------------------------------------------
// Row of sorted position p is rows[perm[p] / k].  mean: divide each cluster's sum by its member count.
// partial: 2 * ceil(N / kCentroidWindow) rows of d binary32 sums; counters: as many counts, zero on entry
// (launch_group clears them).
hipError_t launch_centroid(const void* rows, const int32_t* perm, const int32_t* seg_offsets, const int32_t* seg_of,
                           const int32_t* num_segments, void* centroids, float* partial, uint32_t* counters, int64_t N,
                           int k, int d, bool bf16, bool mean, hipStream_t stream);

// ---- step 4: restore ----------------------------------------------------
// perm and num_segments (both optional): allow the kernel to walk the rows in cluster order when clusters are long.
hipError_t launch_restore(const void* tokens, const void* centroids, const void* expert_out,
                          const int32_t* seg_of, const int32_t* seg_offsets, const int32_t* perm,
                          const int32_t* num_segments, void* out, int64_t N, int k, int d, bool bf16, uint32_t flags,
                          hipStream_t stream);

hipError_t launch_restore_combine(const void* tokens, const void* centroids, const void* expert_out,
                                  const int32_t* seg_of, const int32_t* seg_offsets, const float* gate_weight,
                                  void* out, int64_t T, int k, int d, bool bf16, uint32_t flags, hipStream_t stream);

// ---- backward of steps 3 and 4 -------------------------------------------
struct BackwardPlan {
  size_t windows;  // window sums / counters of the segment sum
  size_t off_partial, off_counters, total_bytes;
};
BackwardPlan plan_backward(int64_t N, int d);
hipError_t launch_clear_counters(uint32_t* counters, size_t n, hipStream_t stream);
hipError_t launch_grad_tokens(const void* grad_out, const void* grad_centroids, const void* grad_expert_out,
                              const int32_t* seg_of, const int32_t* seg_offsets, void* grad_tokens, int64_t T, int k,
                              int d, bool bf16, uint32_t flags, hipStream_t stream);

// Backward of the fused restore + combine: grad_w [T][k] binary32, grad_rows [T][k][d] in the storage type.
hipError_t launch_combine_backward(const void* tokens, const void* centroids, const void* expert_out,
                                   const int32_t* seg_of, const int32_t* seg_offsets, const float* gate_weight,
                                   const void* grad_out, float* grad_w, void* grad_rows, int64_t T, int k, int d, bool bf16,
                                   uint32_t flags, hipStream_t stream);

}  // namespace lshmoe
