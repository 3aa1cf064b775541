// Cross-polytope hash (Section 3.2, Eq. 3) as an MFMA GEMM with the signed
// argmax taken from the accumulator registers.
//
// The product is arranged as Y^T = R * X^T so that, in the 32x32 MFMA
// accumulator layout, a lane holds 16 of the 32 rotated coordinates of ONE
// token (accumulator register j of lane l is row 8*(j/4) + 4*(l/32) + j%4,
// column l%32).  The arg-max over the r coordinates of a hash is then a scan
// over a lane's own registers plus one exchange with lane l^32; the rotated
// vectors are never written to memory.
//
// Both MFMA operands take 8 (bf16) or 1 (fp32) consecutive k values per lane
// with the same (lane, element) -> k mapping, so which k a lane fetches is
// free as long as A and B agree: every lane fetches one 16-byte piece of its
// row per step.
#include "kernels.h"

namespace lshmoe {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename DT> struct Frag;

template <> struct Frag<BF16> {
  static constexpr int kStepElems = 16;  // k values consumed per step by the two lane halves together
  static constexpr int kLaneElems = 8;
  uint4 q;
  __device__ __forceinline__ void load(const char* row, int elem, int d) {
    q = elem < d ? *reinterpret_cast<const uint4*>(row + (size_t)elem * 2) : make_uint4(0, 0, 0, 0);
  }
  static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.q), __builtin_bit_cast(bf16x8, b.q), c,
                                                0, 0, 0);
  }
};

template <> struct Frag<F32> {
  static constexpr int kStepElems = 8;
  static constexpr int kLaneElems = 4;
  float4 q;
  __device__ __forceinline__ void load(const char* row, int elem, int d) {
    q = elem < d ? *reinterpret_cast<const float4*>(row + (size_t)elem * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.q.x, b.q.x, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.q.y, b.q.y, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.q.z, b.q.z, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.q.w, b.q.w, c, 0, 0, 0);
  }
};

// One wave hashes 32 tokens.  The L hashes are processed in groups of `hpg`
// whole hashes (hpg * r <= 32 * NT rows of R per group).
template <typename DT, int NT>
__global__ __launch_bounds__(256) void hash_kernel(const char* __restrict__ tokens, const char* __restrict__ rot,
                                                   uint64_t* __restrict__ bucket, uint32_t T, int d, int L, int r,
                                                   int hpg) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, h = lane >> 5;
  const uint32_t token0 = (blockIdx.x * 4u + wave) * 32u;
  if (token0 >= T) return;
  const uint32_t tok = min(token0 + n, T - 1);
  const size_t row_bytes = (size_t)d * Chunk<DT>::kItem;
  const char* xrow = tokens + (size_t)tok * row_bytes;
  uint64_t b = 0;

  for (int l0 = 0; l0 < L; l0 += hpg) {
    const int nh = min(hpg, L - l0);
    const int rows = nh * r;
    const char* arow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) arow[t] = rot + (size_t)(l0 * r + min(t * 32 + n, rows - 1)) * row_bytes;
    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[t][j] = 0.0f;

    for (int kk = 0; kk < d; kk += Frag<DT>::kStepElems) {
      const int elem = kk + h * Frag<DT>::kLaneElems;
      Frag<DT> fb;
      fb.load(xrow, elem, d);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        Frag<DT> fa;
        fa.load(arow[t], elem, d);
        Frag<DT>::mma(fa, fb, acc[t]);
      }
    }

    for (int lh = 0; lh < nh; ++lh) {
      const int lo = lh * r, hi = lo + r;
      float best = -1.0f;
      int bi = 0x7fffffff;
      bool neg = false;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        if (t * 32 + 31 < lo || t * 32 >= hi) continue;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int mr = t * 32 + 8 * (j >> 2) + 4 * h + (j & 3);  // ascending in j for a fixed lane
          const float v = acc[t][j];
          const float av = fabsf(v);
          if (mr >= lo && mr < hi && av > best) {
            best = av;
            bi = mr - lo;
            neg = v < 0.0f;
          }
        }
      }
      const float obest = __shfl_xor(best, 32, 64);
      const int obi = __shfl_xor(bi, 32, 64);
      const int oneg = __shfl_xor((int)neg, 32, 64);
      if (obest > best || (obest == best && obi < bi)) {
        bi = obi;
        neg = oneg != 0;
      }
      b = b * (uint64_t)(2 * r) + (uint64_t)(bi + (neg ? r : 0));
    }
  }
  if (h == 0 && token0 + n < T) bucket[token0 + n] = b;
}

template <typename DT>
hipError_t launch_typed(const void* tokens, const void* rot, int64_t T, int d, int L, int r, uint64_t* bucket,
                        hipStream_t stream) {
  int hpg = 256 / r;
  if (hpg > L) hpg = L;
  if (hpg < 1) return hipErrorInvalidValue;
  const int nt = (hpg * r + 31) / 32;
  const dim3 grid((uint32_t)((T + 127) / 128)), block(256);
  auto x = (const char*)tokens;
  auto R = (const char*)rot;
#define LSHMOE_HASH_CASE(NT)                                                                                   \
  hipLaunchKernelGGL((hash_kernel<DT, NT>), grid, block, 0, stream, x, R, bucket, (uint32_t)T, d, L, r, hpg)
  if (nt <= 1) LSHMOE_HASH_CASE(1);
  else if (nt == 2) LSHMOE_HASH_CASE(2);
  else if (nt == 3) LSHMOE_HASH_CASE(3);
  else if (nt == 4) LSHMOE_HASH_CASE(4);
  else if (nt <= 6) LSHMOE_HASH_CASE(6);
  else LSHMOE_HASH_CASE(8);
#undef LSHMOE_HASH_CASE
  return hipGetLastError();
}

}  // namespace

hipError_t launch_hash(const void* tokens, const void* rot, int64_t T, int d, int L, int r, bool bf16,
                       uint64_t* bucket, hipStream_t stream) {
  return bf16 ? launch_typed<BF16>(tokens, rot, T, d, L, r, bucket, stream)
              : launch_typed<F32>(tokens, rot, T, d, L, r, bucket, stream);
}

}  // namespace lshmoe
