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

// One 16-byte chunk of a row, widened to binary32 lanes.
template <typename DT> struct Chunk;

template <> struct Chunk<F32> {
  static constexpr int kElems = 4;
  static constexpr int kItem = 4;
  float v[4];
  __device__ __forceinline__ void load(const void* row, int chunk) {
    const float4 q = reinterpret_cast<const float4*>(row)[chunk];
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
  }
  __device__ __forceinline__ void store(void* row, int chunk) const {
    reinterpret_cast<float4*>(row)[chunk] = make_float4(v[0], v[1], v[2], v[3]);
  }
};

template <> struct Chunk<BF16> {
  static constexpr int kElems = 8;
  static constexpr int kItem = 2;
  float v[8];
  __device__ __forceinline__ void load(const void* row, int chunk) {
    const uint4 q = reinterpret_cast<const uint4*>(row)[chunk];
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ __forceinline__ void store(void* row, int chunk) const {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f32_to_bf16_bits(v[2 * i]) | (f32_to_bf16_bits(v[2 * i + 1]) << 16);
    reinterpret_cast<uint4*>(row)[chunk] = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

}  // namespace lshmoe
