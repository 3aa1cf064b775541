// Measured-peak probes for the benchmark's roofline context: what this GPU sustains for a pure streaming read,
// a streaming copy, and a loop of independent bf16 MFMAs.  Not part of the compression path and not part of its
// ABI: bench.py --peaks loads this small library on its own.
//
// All pointers are device pointers owned by the caller; every call only enqueues work on `stream`.
#include <hip/hip_runtime.h>
#include <cstdint>

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Every workgroup owns whole tiles of kUnroll x 256 consecutive 16-byte pieces (kUnroll x 4 KB) and walks them
// with a grid stride; a thread has kUnroll pieces in flight.
constexpr int kUnroll = 8;

__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, size_t pieces, uint32_t* sink) {
  const size_t tile = (size_t)kUnroll * 256, tiles = pieces / tile;
  uint32_t acc = 0;
  for (size_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const uint4* p = src + t * tile + threadIdx.x;
    uint4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = p[u * 256];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= v[u].x ^ v[u].w;
  }
  for (size_t i = tiles * tile + (size_t)blockIdx.x * 256 + threadIdx.x; i < pieces; i += (size_t)gridDim.x * 256) acc ^= src[i].x;
  if (acc == 0x9e3779b9u) *sink = acc;   // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t pieces) {
  const size_t tile = (size_t)kUnroll * 256, tiles = pieces / tile;
  for (size_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const uint4* p = src + t * tile + threadIdx.x;
    uint4* q = dst + t * tile + threadIdx.x;
    uint4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = p[u * 256];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const u32x4 w = {v[u].x, v[u].y, v[u].z, v[u].w};
      __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(q + u * 256));
    }
  }
  for (size_t i = tiles * tile + (size_t)blockIdx.x * 256 + threadIdx.x; i < pieces; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// four independent accumulator chains per wave, no memory traffic inside the loop
__global__ __launch_bounds__(256) void mfma_kernel(float* out, int iters) {
  floatx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[t][j] = 0.0f;
  const uint4 qa = make_uint4(threadIdx.x, 1, 2, 3), qb = make_uint4(5, threadIdx.x, 7, 8);
  const bf16x8 a = __builtin_bit_cast(bf16x8, qa), b = __builtin_bit_cast(bf16x8, qb);
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[t][j];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// The same loop on operands that differ from one MFMA to the next: eight fragment pairs of random bf16 values of
// magnitude about one, read once from `operands` (64 lanes x 16 pieces of 16 bytes per workgroup wave, the same for
// every wave) and cycled through.  The matrix cores draw more power on such data than on constants, and the
// clock they sustain is lower: this is the rate a GEMM on real data can hope for.
__global__ __launch_bounds__(256) void mfma_random_kernel(const uint4* __restrict__ operands, float* out, int iters) {
  floatx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[t][j] = 0.0f;
  const int lane = threadIdx.x & 63;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    a[q] = __builtin_bit_cast(bf16x8, operands[(2 * q) * 64 + lane]);
    b[q] = __builtin_bit_cast(bf16x8, operands[(2 * q + 1) * 64 + lane]);
  }
  for (int i = 0; i < iters; i += 2) {   // two rounds per pass: every MFMA of a pass has operands of its own
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[4 * r + t], b[4 * r + t], acc[t], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[t][j];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" {

// Reads `bytes` (a multiple of 16) from src once with `blocks` workgroups.  sink: 4 bytes of device memory.
// Returns 0 or a hipError_t.
int peaks_read(const void* src, size_t bytes, void* sink, int blocks, void* stream) {
  if (src == nullptr || sink == nullptr || bytes % 16 != 0 || blocks <= 0) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(read_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, bytes / 16,
                     (uint32_t*)sink);
  return (int)hipGetLastError();
}

// Copies `bytes` (a multiple of 16) from src to dst (no overlap) with streaming stores.
int peaks_copy(const void* src, void* dst, size_t bytes, int blocks, void* stream) {
  if (src == nullptr || dst == nullptr || bytes % 16 != 0 || blocks <= 0) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst,
                     bytes / 16);
  return (int)hipGetLastError();
}

// Runs blocks x 4 waves x iters x 4 v_mfma_f32_32x32x16_bf16 (32768 flop each); out: blocks * 256 floats.
int peaks_mfma_bf16(int blocks, int iters, float* out, void* stream) {
  if (out == nullptr || blocks <= 0 || iters <= 0) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(mfma_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters);
  return (int)hipGetLastError();
}

// The same count of MFMAs on changing operands.  operands: 16 x 64 pieces of 16 bytes (16 KB) of device memory
// holding bf16 values; iters must be even.
int peaks_mfma_bf16_random(const void* operands, int blocks, int iters, float* out, void* stream) {
  if (operands == nullptr || out == nullptr || blocks <= 0 || iters <= 0 || iters % 2 != 0) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(mfma_random_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)operands, out,
                     iters);
  return (int)hipGetLastError();
}

}  // extern "C"
