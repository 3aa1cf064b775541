// Shared device helpers for the gfx950 kernels: storage-type traits and
// 16-byte vector access.  Wavefront size is 64 throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lshmoe {

constexpr int kWave = 64;

struct F32 {};   // IEEE binary32 storage
struct BF16 {};  // bfloat16 storage (upper half of binary32)

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// binary32 -> bfloat16, round to nearest even on the 16 discarded bits.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// One wave per row (or cluster) can mean more than 2^32 threads, which a one-dimensional launch cannot express
// (a dispatch counts work-items per dimension in 32 bits): grids of 256-thread workgroups beyond 2^22 workgroups
// are folded into two dimensions.  Surplus workgroups of the last row leave through the kernels' bounds checks.
inline dim3 grid_of_blocks(uint64_t blocks) {
  constexpr uint64_t kMaxX = 1ull << 22;
  if (blocks <= kMaxX) return dim3((uint32_t)(blocks == 0 ? 1 : blocks));
  const uint64_t by = (blocks + kMaxX - 1) / kMaxX;
  return dim3((uint32_t)((blocks + by - 1) / by), (uint32_t)by);
}
__device__ __forceinline__ uint64_t linear_block() { return (uint64_t)blockIdx.y * gridDim.x + blockIdx.x; }

// Rows are moved as raw 16-byte pieces (uint4) and only widened to binary32
// where arithmetic happens, so that loads in flight cost 4 registers each.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 load16(const char* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void store16(char* p, uint4 v) { *reinterpret_cast<uint4*>(p) = v; }
// Streaming store: the line is not kept in the caches (outputs that nobody in this kernel reads again).
__device__ __forceinline__ void store16_stream(char* p, uint4 v) {
  const u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(p));
}

template <typename DT> struct Piece;   // arithmetic on one 16-byte piece

template <> struct Piece<F32> {
  static constexpr int kElems = 4;
  static __device__ __forceinline__ void widen(uint4 q, float (&v)[4]) {
    v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y); v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w);
  }
  static __device__ __forceinline__ uint4 narrow(const float (&v)[4]) {
    return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
  }
};

template <> struct Piece<BF16> {
  static constexpr int kElems = 8;
  static __device__ __forceinline__ void widen(uint4 q, float (&v)[8]) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ uint4 narrow(const float (&v)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f32_to_bf16_bits(v[2 * i]) | (f32_to_bf16_bits(v[2 * i + 1]) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
};

template <typename DT> struct ItemSize;
template <> struct ItemSize<F32> { static constexpr int value = 4; };
template <> struct ItemSize<BF16> { static constexpr int value = 2; };

}  // namespace lshmoe
