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
// Tiling.  A workgroup of WAVES waves owns WAVES*NTK*32 tokens and all rows of one
// "hash group" (as many whole hashes as fit in 256 rows of R).  Each wave
// keeps MT x NTK accumulator tiles (all rows, its own NTK*32 tokens), so a
// token's bucket id is completed inside one wave.  k is walked in chunks of
// 128 bytes per row (4 MFMA steps).
//
//   tokens (B operand): the MFMA B layout wants, per lane, 16 bytes of one
//     token's row.  Lanes fetch exactly that from global memory, straight
//     into registers, XDEPTH-1 chunks ahead of use; measured on MI355X this
//     access streams as fast as a fully coalesced read, so the tokens - the
//     only HBM traffic of the kernel - never touch LDS.
//   R (A operand): shared by the waves, so each 128-byte chunk of the
//     group's rows is staged in LDS (double buffered; the next chunk's global
//     loads are in flight during the MFMAs of the current one).  The rows sit
//     in LDS with an XOR swizzle of the 16-byte piece index by the row so
//     that the fragment reads of 8 consecutive rows hit 8 different bank
//     groups (measured: full 128 B/clk) while global loads stay coalesced.
//
// Both MFMA operands take their k values with the same (lane, element) -> k
// mapping, so which k a lane supplies is free as long as A and B agree: the
// lane half h = l/32 takes piece 2s + h of the chunk in step s.
#include <atomic>
#include <utility>

#include "kernels.h"

namespace lshmoe {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename DT> struct Mma;

template <> struct Mma<BF16> {
  static __device__ __forceinline__ void run(const uint4& a, const uint4& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

template <> struct Mma<F32> {
  static __device__ __forceinline__ void run(const uint4& a, const uint4& b, floatx16& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
  }
};

constexpr int kPieces = 8;   // 16-byte pieces per row per chunk
constexpr int kSteps = 4;    // MFMA steps per chunk (two pieces, one per lane half, per step)

__device__ __forceinline__ int swizzle(int row, int piece) { return piece ^ (row & 7); }

// Compile-time loop: f is called with std::integral_constant<int, 0> .. <int, N - 1>, so that every index derived
// from it is a constant expression.
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Arg-max of |y| over the rows a lane holds of one hash whose rows are the NT whole 32-row tiles T0 .. T0 + NT - 1 of
// the lane's accumulators, for NTW token tiles at once (their chains are independent, which keeps the vector unit
// busy).  One pass in ascending row order: a strictly larger magnitude replaces the candidate, so the lowest row
// wins among equal magnitudes; the candidate starts as +0 at the lane's first row.  bv: value at the candidate;
// bid: its row inside the hash, without the lane half's offset of 4 rows.
template <int T0, int NT, int MTW, int NTW>
__device__ __forceinline__ void scan_hash_tiles(const floatx16 (&acc)[MTW][NTW], float (&bv)[NTW], int (&bid)[NTW]) {
  static_for<NTW>([&](auto uc) {
    bv[decltype(uc)::value] = 0.0f;
    bid[decltype(uc)::value] = 0;
  });
  static_for<NT * 16>([&](auto qc) {
    constexpr int q = decltype(qc)::value;
    constexpr int t = q / 16, j = q % 16;            // register j of tile T0 + t: row 32 t + 8 (j / 4) + 4 h + j % 4
    static_for<NTW>([&](auto uc) {
      constexpr int u = decltype(uc)::value;
      const float v = acc[T0 + t][u][j];
      if (fabsf(v) > fabsf(bv[u])) {
        bv[u] = v;
        bid[u] = 32 * t + 8 * (j / 4) + j % 4;
      }
    });
  });
}

// Joins a lane's candidate with that of lane ^ 32, which holds the other 16 rows of every tile.  Returns the
// magnitude pattern; row and sign of the winner are left in bi and neg.  -0 counts as positive.
__device__ __forceinline__ uint32_t join_lane_halves(float bv, int& bi, bool& neg) {
  uint32_t best = __float_as_uint(bv) & 0x7fffffffu;
  neg = (__float_as_uint(bv) >> 31) != 0u && best != 0u;
  const uint32_t obest = (uint32_t)__shfl_xor((int)best, 32, 64);
  const int obi = __shfl_xor(bi, 32, 64);
  const int oneg = __shfl_xor((int)neg, 32, 64);
  if (obest > best || (obest == best && obi < bi)) {
    best = obest;
    bi = obi;
    neg = oneg != 0;
  }
  return best;
}

// Sum of the squares of the elements of one 16-byte piece, added to acc in element order.
template <typename DT> __device__ __forceinline__ float add_squares(const uint4& q, float acc) {
  float v[Piece<DT>::kElems];
  Piece<DT>::widen(q, v);
#pragma unroll
  for (int i = 0; i < Piece<DT>::kElems; ++i) acc = fmaf(v[i], v[i], acc);
  return acc;
}

// SPHERE: the rows of `rot` are the pivots of r spheres (L = 1, one pass) and the code is one bit per sphere instead
// of an arg-max: bit i = [ |x|^2 - 2 <p_i, x> + |p_i|^2 <= radius_sq[i] ], bit 0 most significant.  The dot products
// are the same MFMA product; |x|^2 is gathered from the token pieces a lane feeds to the MFMAs (the two lane halves
// hold the two halves of every chunk) and |p_i|^2 from the pieces a thread stages, all in binary32.
template <typename DT, int MT, int NTK, int XDEPTH, int WAVES, int OCC, bool ALIGNED8, bool KTAIL, bool SPHERE = false>
__global__ __launch_bounds__(WAVES * 64, OCC) void hash_kernel(const char* __restrict__ tokens, const char* __restrict__ rot,
                                                   uint64_t* __restrict__ bucket, uint32_t T, int row_pieces, int L,
                                                   int r, int hpg, const float* __restrict__ radius_sq = nullptr) {
  constexpr int RA = MT * 32;              // rows of R staged per chunk
  constexpr int SLOTS = RA * kPieces;      // 16-byte slots per LDS buffer
  extern __shared__ uint4 lds[];           // [2][SLOTS]

  const int tid = threadIdx.x;
  constexpr int TH = WAVES * 64;           // threads of the workgroup
  constexpr int RS = TH / kPieces;         // rows of R one staging sweep of the workgroup covers
  constexpr int LA = RA / RS;              // staging loads per thread and chunk
  static_assert(RA % RS == 0, "the rows of R must be a whole number of staging sweeps");
  __builtin_assume(tid >= 0 && tid < TH);
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const uint32_t row_bytes = (uint32_t)row_pieces * 16u;
  const int nchunks = ((row_pieces + kPieces - 1) / kPieces + XDEPTH - 1) / XDEPTH * XDEPTH;

  // token rows of this lane (rows past the last token re-read it; their ids are never stored)
  const uint32_t tok_wave = (blockIdx.x * (uint32_t)WAVES + wave) * (uint32_t)(NTK * 32);
  const char* xrow[NTK];
#pragma unroll
  for (int u = 0; u < NTK; ++u)
    xrow[u] = tokens + (size_t)min(tok_wave + (uint32_t)(u * 32 + n), T - 1) * row_bytes + h * 16;

  // R staging: this thread always moves piece lp of rows r0, r0 + 32, ...
  const int lp = tid & 7, r0 = tid >> 3;
  const int st_slot = r0 * kPieces + swizzle(r0, lp);  // row offsets that are multiples of 8 keep the swizzle
  int fa_slot[kSteps];
#pragma unroll
  for (int s = 0; s < kSteps; ++s) fa_slot[s] = n * kPieces + swizzle(n, 2 * s + h);

  uint64_t b[NTK];
#pragma unroll
  for (int t = 0; t < NTK; ++t) b[t] = 0;

  for (int l0 = 0; l0 < L; l0 += hpg) {
    const int nh = min(hpg, L - l0);
    const int rows = nh * r;               // valid rows of R in this group (<= RA); rows past them repeat the last
    const char* rot_group = rot + (size_t)l0 * r * row_bytes;
    uint32_t off_a[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) off_a[i] = (uint32_t)min(r0 + i * RS, rows - 1) * row_bytes + lp * 16;

    uint4 stage[LA];
    auto load_r = [&](int chunk) {
      const bool in_row = !KTAIL || chunk * kPieces + lp < row_pieces;   // the k tail is zero filled
      const char* a_base = rot_group + (size_t)chunk * (kPieces * 16);
#pragma unroll
      for (int i = 0; i < LA; ++i)
        stage[i] = in_row ? *reinterpret_cast<const uint4*>(a_base + off_a[i]) : make_uint4(0, 0, 0, 0);
    };
    float pn[LA], nx2[NTK];                // SPHERE: partial |p|^2 of the rows this thread stages, partial |x|^2
#pragma unroll
    for (int i = 0; i < LA; ++i) pn[i] = 0.0f;
#pragma unroll
    for (int u = 0; u < NTK; ++u) nx2[u] = 0.0f;
    auto store_r = [&](int buf) {
      uint4* dst = lds + buf * SLOTS + st_slot;
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        dst[i * TH] = stage[i];
        if (SPHERE) pn[i] = add_squares<DT>(stage[i], pn[i]);
      }
    };
    uint4 xr[XDEPTH][NTK][kSteps];
    auto load_x = [&](int chunk, uint4 (&dst)[NTK][kSteps]) {
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const bool in_row = !KTAIL || chunk * kPieces + 2 * s + h < row_pieces;
#pragma unroll
        for (int u = 0; u < NTK; ++u)
          dst[u][s] = in_row ? *reinterpret_cast<const uint4*>(xrow[u] + (size_t)chunk * (kPieces * 16) + s * 32)
                             : make_uint4(0, 0, 0, 0);
      }
    };

    floatx16 acc[MT][NTK];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int u = 0; u < NTK; ++u)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[t][u][j] = 0.0f;

    __syncthreads();                       // previous group's readers are done with both buffers
    load_r(0);
#pragma unroll
    for (int j = 0; j < XDEPTH - 1; ++j)
      if (j < nchunks) load_x(j, xr[j]);
    store_r(0);
    __syncthreads();

    // nchunks is a multiple of XDEPTH (the host rounds it up; with KTAIL the surplus chunks read as zeros),
    // so the unrolled body needs no early exit and the accumulators stay in place
    for (int c0 = 0; c0 < nchunks; c0 += XDEPTH) {
#pragma unroll
      for (int j = 0; j < XDEPTH; ++j) {
        const int c = c0 + j;
        const bool more = c + 1 < nchunks;
        if (more) load_r(c + 1);
        if (c + XDEPTH - 1 < nchunks) load_x(c + XDEPTH - 1, xr[(j + XDEPTH - 1) % XDEPTH]);
        const uint4* buf = lds + (c & 1) * SLOTS;
        if (SPHERE) {
#pragma unroll
          for (int u = 0; u < NTK; ++u)
#pragma unroll
            for (int st = 0; st < kSteps; ++st) nx2[u] = add_squares<DT>(xr[j][u][st], nx2[u]);
        }
        // A fragments go through a small ring: the LDS read of (step, tile) i + kAhead is issued before the
        // MFMAs of (step, tile) i, and the scheduler is told to keep that order
        constexpr int kAhead = 3, kRing = 4, kFrags = kSteps * MT;
        uint4 fa[kRing];
#pragma unroll
        for (int i = 0; i < kAhead && i < kFrags; ++i) fa[i] = buf[fa_slot[i / MT] + (i % MT) * 32 * kPieces];
#pragma unroll
        for (int i = 0; i < kFrags; ++i) {
          if (i + kAhead < kFrags)
            fa[(i + kAhead) % kRing] = buf[fa_slot[(i + kAhead) / MT] + ((i + kAhead) % MT) * 32 * kPieces];
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < NTK; ++u) Mma<DT>::run(fa[i % kRing], xr[j][u][i / MT], acc[i % MT][u]);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (more) store_r((c + 1) & 1);
        __syncthreads();
      }
    }

    if (SPHERE) {
      // |p_i|^2: the 8 threads that staged the 8 pieces of a row sit in 8 consecutive lanes
      float* pn2 = reinterpret_cast<float*>(lds);   // [RA]; every wave is past the last chunk's closing barrier
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        float v = pn[i];
        v += __shfl_xor(v, 1, 64);
        v += __shfl_xor(v, 2, 64);
        v += __shfl_xor(v, 4, 64);
        if (lp == 0) pn2[r0 + i * RS] = v;
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < NTK; ++u) {
        const float xx = nx2[u] + __shfl_xor(nx2[u], 32, 64);
        uint64_t bits = 0;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const int row = t * 32 + 8 * (j >> 2) + 4 * h + (j & 3);
            if (row < r) {
              const float dist2 = (xx - 2.0f * acc[t][u][j]) + pn2[row];
              if (dist2 <= radius_sq[row]) bits |= 1ull << (r - 1 - row);
            }
          }
        }
        const uint32_t lo32 = (uint32_t)bits, hi32 = (uint32_t)(bits >> 32);
        bits |= (uint64_t)(uint32_t)__shfl_xor((int)lo32, 32, 64) | ((uint64_t)(uint32_t)__shfl_xor((int)hi32, 32, 64) << 32);
        b[u] = bits;
      }
      continue;   // one pass (hpg = L = 1)
    }
    // signed arg-max per hash of the group, from the accumulators
#pragma unroll
    for (int u = 0; u < NTK; ++u) {
      for (int lh = 0; lh < nh; ++lh) {
        const int lo = lh * r;
        uint32_t best;   // bit pattern of the largest magnitude among this lane's rows of the hash
        int bi;          // lowest row (relative to the hash) attaining it
        bool neg;        // sign of the value there
        if (ALIGNED8) {
          // r and every hash boundary are multiples of 8: the four rows 8*jb + 4*h + (0..3) a lane holds of
          // an 8-row block are inside the hash or outside it together, for every lane alike.
          // Pass 1: binary32 patterns order like integers, so a signed-integer max finds the largest positive
          // value and an unsigned max the largest-magnitude negative one (two 3-operand max chains).
          int pmax = (int)0x80000000;
          uint32_t nmax = 0;
#pragma unroll
          for (int t = 0; t < MT; ++t) {
            if (t * 32 + 31 < lo || t * 32 >= lo + r) continue;  // wave-uniform
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
              const int base = t * 32 + 8 * jb - lo;
              if (base < 0 || base >= r) continue;  // wave-uniform
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const uint32_t vi = __float_as_uint(acc[t][u][4 * jb + i]);
                pmax = max(pmax, (int)vi);
                nmax = max(nmax, vi);
              }
            }
          }
          const uint32_t mp = pmax >= 0 ? (uint32_t)pmax : 0u;
          const uint32_t mn = (nmax >> 31) ? (nmax & 0x7fffffffu) : 0u;
          best = max(mp, mn);
          neg = mn > mp;
          // Pass 2: lowest row whose magnitude equals the maximum (descending, so the last hit is the lowest).
          const float bestf = __uint_as_float(best);
          bi = 0x7fffffff;
#pragma unroll
          for (int t = MT - 1; t >= 0; --t) {
            if (t * 32 + 31 < lo || t * 32 >= lo + r) continue;
#pragma unroll
            for (int jb = 3; jb >= 0; --jb) {
              const int base = t * 32 + 8 * jb - lo;
              if (base < 0 || base >= r) continue;
#pragma unroll
              for (int i = 3; i >= 0; --i)
                if (fabsf(acc[t][u][4 * jb + i]) == bestf) bi = base + 4 * h + i;
            }
          }
          // +m and -m both present in this lane (exact tie in magnitude): the sign is that of the lowest row
          if (__any(mp == mn && best != 0u)) {
            uint32_t wbits = neg ? 0x80000000u : 0u;  // pattern of the value at the lowest such row
#pragma unroll
            for (int t = MT - 1; t >= 0; --t) {
              if (t * 32 + 31 < lo || t * 32 >= lo + r) continue;
#pragma unroll
              for (int jb = 3; jb >= 0; --jb) {
                const int base = t * 32 + 8 * jb - lo;
                if (base < 0 || base >= r) continue;
#pragma unroll
                for (int i = 3; i >= 0; --i) {
                  const float v = acc[t][u][4 * jb + i];
                  if (fabsf(v) == bestf) wbits = __float_as_uint(v);
                }
              }
            }
            neg = (wbits >> 31) != 0u;
          }
        } else {
          float bestf = -1.0f, bv = 0.0f;
          bi = 0x7fffffff;
#pragma unroll
          for (int t = 0; t < MT; ++t) {
            if (t * 32 + 31 < lo || t * 32 >= lo + r) continue;  // wave-uniform
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              const int rel = t * 32 + 8 * (j >> 2) + 4 * h + (j & 3) - lo;  // ascending in j for a fixed lane
              const float v = acc[t][u][j];
              const float av = (unsigned)rel < (unsigned)r ? fabsf(v) : -2.0f;
              if (av > bestf) {
                bestf = av;
                bi = rel;
                bv = v;
              }
            }
          }
          best = bestf < 0.0f ? 0u : __float_as_uint(bestf);  // a lane may hold no row of this hash
          neg = bv < 0.0f;
        }
        // the other half of the token's rows sits in lane l ^ 32 (magnitude patterns compare as integers)
        const uint32_t obest = (uint32_t)__shfl_xor((int)best, 32, 64);
        const int obi = __shfl_xor(bi, 32, 64);
        const int oneg = __shfl_xor((int)neg, 32, 64);
        if (obest > best || (obest == best && obi < bi)) {
          bi = obi;
          neg = oneg != 0;
        }
        b[u] = b[u] * (uint64_t)(2 * r) + (uint64_t)(bi + (neg ? r : 0));
      }
    }
  }
  if (h == 0) {
#pragma unroll
    for (int u = 0; u < NTK; ++u) {
      const uint32_t tok = tok_wave + (uint32_t)(u * 32 + n);
      if (tok < T) bucket[tok] = b[u];
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Streaming variant: BOTH operands are staged through LDS by direct global->LDS loads, several chunks ahead.
//
// Why.  In hash_kernel the tokens go straight into registers: 32 bytes of 32 different rows per load
// instruction, which loads the address path, and with eight 32-row tiles and one 32-token tile per wave
// every MFMA needs a fresh A fragment from LDS, which is exactly the LDS read peak (1 KB per 32-cycle MFMA
// and SIMD).  Here the token rows are fetched as whole 128-byte lines (8 lanes per row), need no staging
// registers and no LDS write instructions, and a wave keeps MTW x NTW tiles, so that with NTW = 2 a wave
// reads MTW + 2 fragments for 2*MTW MFMAs.
//
// Shape.  A workgroup has GROUPS token groups of NTW*32 tokens and, for the widest hash groups, HALVES = 2
// waves per token group that each hold half of the rows of R (two waves sharing a token group read the
// tokens from LDS, not twice from memory); their results are joined at the end through LDS.
//
// Staging.  Chunk c (128 bytes of every row) of R sits in slot c % (DR + 1) of a ring, of the tokens in slot
// c % (DX + 1); iteration c issues the loads of R chunk c + DR and token chunk c + DX (R from L2, the tokens
// from HBM, hence the longer distance).  The loads of a wave complete in issue order, so "chunk c + 1 has
// landed" is a wait until at most kAllowed of the wave's loads are in flight, followed by the barrier that
// closes the iteration.
// Requires: r a multiple of 8, rows a whole number of 128-byte chunks.
//
// 16 bytes per lane straight from global memory into LDS: lane l's piece lands at dst + l (dst is wave-uniform).
// Written as inline assembly on purpose: for the compiler's own builtin the wait-count pass holds every later
// LDS read until the load has landed, which would serialise the staging with the MFMA loop.  The caller
// waits for these loads itself (s_waitcnt vmcnt) before the barrier that publishes the buffer.
__device__ __forceinline__ void load16_to_lds(const char* src, uint4* dst) {
  const uint32_t lds_addr = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)dst);
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "memory", "m0");
}

// s_waitcnt until at most n vector-memory operations of the wave are in flight (LDS and scalar counters untouched).
template <int N> __device__ __forceinline__ void wait_vm_at_most() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

template <int MTW, int NTW, int GROUPS, int HALVES, int DR, int DX> struct StreamShape {
  static constexpr int kWaves = GROUPS * HALVES;
  static constexpr int kRows = MTW * HALVES * 32;    // rows of R staged per chunk
  static constexpr int kTokens = GROUPS * NTW * 32;  // tokens of a workgroup
  static constexpr int kSlotsR = kRows * kPieces, kSlotsX = kTokens * kPieces;  // 16-byte slots per ring slot
  static constexpr size_t kLdsBytes = ((size_t)(DR + 1) * kSlotsR + (size_t)(DX + 1) * kSlotsX) * 16;
};

// GATE: E further rows (a gate projection W_g, same layout as R) are appended to the rows of the single hash
// group; their products are written to logits[T][E] as binary32 instead of entering an arg-max, so that the
// hash and the gate read the tokens once.  L = 0 computes the gate rows alone.
// RC: 0, or the value of r when it is 32, 64, 128 or 256 and hash boundaries fall on tile boundaries of every
// wave (the launcher checks): the arg-max then runs over compile-time row ranges, without a branch per block of
// rows; it is a quarter to a third of the generic one's time, which at the largest shapes was a sixth of the kernel.
template <typename DT, int MTW, int NTW, int GROUPS, int HALVES, int DR, int DX, bool GATE = false, int RC = 0>
__global__ __launch_bounds__(GROUPS * HALVES * 64, 1) void hash_stream_kernel(
    const char* __restrict__ tokens, const char* __restrict__ rot, uint64_t* __restrict__ bucket, uint32_t T,
    int row_pieces, int L, int r, int hpg, const char* __restrict__ gate_w = nullptr, int E = 0,
    float* __restrict__ logits = nullptr) {
  using S = StreamShape<MTW, NTW, GROUPS, HALVES, DR, DX>;
  // GATE with two halves: each wave's last tile is a tile of gate rows, its first MTW - 1 tiles are rows of R (so
  // that the hashes split between the halves exactly as without the gate).  Staged rows: HALVES * (MTW - 1) tiles
  // of R, then HALVES tiles of gate rows.
  constexpr bool GSPLIT = GATE && HALVES == 2;
  constexpr int MTH = GSPLIT ? MTW - 1 : MTW;   // tiles of rows of R per wave
  static_assert(RC == 0 || ((!GATE || GSPLIT) && (RC == 256 ? (MTH == 4 && HALVES == 2) : (RC % 32 == 0 && (MTH * 32) % RC == 0))),
                "a compile-time r needs whole hashes per wave (or, for r = 256, half a hash)");
  constexpr int WAVES = S::kWaves, TH = WAVES * 64;
  constexpr int LR = S::kRows / 8 / WAVES, LX = S::kTokens / 8 / WAVES;  // direct loads per wave and chunk
  static_assert(S::kRows % (8 * WAVES) == 0 && S::kTokens % (8 * WAVES) == 0, "whole 8-row loads per wave");
  static_assert((DX == DR + 1 || DX == DR) && DR >= 1, "the wait below assumes the tokens run as far ahead as R or one chunk further");
  // loads issued after those of chunk c + 1, at the end of iteration c (iteration i issues R chunk i + DR, then token chunk i + DX)
  constexpr int kAllowed = (DR - 1) * (LR + LX) + (DX == DR + 1 ? LX : 0);
  // The token loads of an iteration come from HBM; a wave that issues them in one burst sits in the issue stage
  // while the memory pipeline is full, its MFMAs waiting behind it.  With two halves (the largest shapes) they are
  // issued a quarter at a time behind the MFMAs of each k step instead; the order of a wave's loads stays R, then
  // tokens, so the wait at the end of the iteration counts as before.
  constexpr bool kSpreadX = HALVES == 2 && DX == DR + 1 && LX >= kSteps;
  extern __shared__ uint4 lds[];             // R ring [DR + 1][kSlotsR], then token ring [DX + 1][kSlotsX]
  const int tid = threadIdx.x;
  __builtin_assume(tid >= 0 && tid < TH);
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int g = wave / HALVES, mh = wave % HALVES;   // token group, half of the rows
  const uint32_t row_bytes = (uint32_t)row_pieces * 16u;
  const int nchunks = row_pieces / kPieces;
  const uint32_t tok_blk = blockIdx.x * (uint32_t)S::kTokens;
  const char* x_blk = tokens + (size_t)tok_blk * row_bytes;

  // a wave's load instruction covers 8 rows x 8 pieces (lane l at slot base + l); the swizzle is applied by
  // choosing which piece of the row a lane fetches
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const int sub = lane >> 3, pc = (lane & 7) ^ sub;  // row inside the 8-row group, logical piece this lane fetches
  uint32_t off_x[LX];
#pragma unroll
  for (int i = 0; i < LX; ++i)               // token rows past the end re-read the last token
    off_x[i] = (min(tok_blk + (uint32_t)(8 * (wv * LX + i) + sub), T - 1) - tok_blk) * row_bytes + pc * 16;
  int fslot[kSteps];
#pragma unroll
  for (int s = 0; s < kSteps; ++s) fslot[s] = n * kPieces + swizzle(n, 2 * s + h);
  const int a_tile0 = mh * MTH * 32 * kPieces;   // first slot of this wave's tiles of R inside an R ring slot
  // slot of the wave's tile t inside an R ring slot (its gate tile, if any, sits behind all tiles of R)
  auto a_tile = [&](int t) { return GSPLIT && t == MTH ? (HALVES * MTH + mh) * 32 * kPieces : a_tile0 + t * 32 * kPieces; };
  const int b_tile0 = g * NTW * 32 * kPieces;    // ... and of its token tiles inside a token ring slot
  uint4* const lds_x = lds + (DR + 1) * S::kSlotsR;

  uint64_t b[NTW];
#pragma unroll
  for (int u = 0; u < NTW; ++u) b[u] = 0;
  for (int l0 = 0; l0 < (GATE ? 1 : L); l0 += hpg) {
    const int nh = GATE ? L : min(hpg, L - l0);
    const int rows_h = nh * r;               // rows of R in this group
    const int rows = rows_h + (GATE ? E : 0);  // valid staged rows; staging rows past them repeat the last
    const char* arow[LR];                    // this lane's piece of the rows it stages (R first, then the gate rows)
#pragma unroll
    for (int i = 0; i < LR; ++i) {
      const int staged = 8 * (wv * LR + i) + sub;
      if (GSPLIT) {                          // tiles of R (rows past the last repeat it), then the tiles of gate rows
        constexpr int kRowsR = HALVES * MTH * 32;
        arow[i] = (staged >= kRowsR ? gate_w + (size_t)min(staged - kRowsR, E - 1) * row_bytes
                                    : rot + (size_t)min(staged, rows_h - 1) * row_bytes) + pc * 16;
      } else {
        const int row = min(staged, rows - 1);
        arow[i] = (GATE && row >= rows_h ? gate_w + (size_t)(row - rows_h) * row_bytes
                                         : rot + ((size_t)l0 * r + row) * row_bytes) + pc * 16;
      }
    }

    auto stage_r = [&](int chunk) {
      uint4* dst = lds + (chunk % (DR + 1)) * S::kSlotsR + (8 * wv * LR) * kPieces;
#pragma unroll
      for (int i = 0; i < LR; ++i) load16_to_lds(arow[i] + (size_t)chunk * (kPieces * 16), dst + 8 * i * kPieces);
    };
    // part s of a token chunk's loads: a quarter of them per k step when the loads are spread over the chunk's steps
    auto stage_x_part = [&](int chunk, int part) {
      uint4* dst = lds_x + (chunk % (DX + 1)) * S::kSlotsX + (8 * wv * LX) * kPieces;
#pragma unroll
      for (int i = 0; i < LX; ++i)
        if (i * kSteps / LX == part) load16_to_lds(x_blk + (size_t)chunk * (kPieces * 16) + off_x[i], dst + 8 * i * kPieces);
    };
    auto stage_x = [&](int chunk) {
      uint4* dst = lds_x + (chunk % (DX + 1)) * S::kSlotsX + (8 * wv * LX) * kPieces;
#pragma unroll
      for (int i = 0; i < LX; ++i) load16_to_lds(x_blk + (size_t)chunk * (kPieces * 16) + off_x[i], dst + 8 * i * kPieces);
    };

    floatx16 acc[MTW][NTW];
#pragma unroll
    for (int t = 0; t < MTW; ++t)
#pragma unroll
      for (int u = 0; u < NTW; ++u)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[t][u][j] = 0.0f;

    __syncthreads();                         // previous group's readers are done with LDS
    // chunks 0 .. DR-1 of R and 0 .. DX-1 of the tokens, in the order the loop would have issued them
#pragma unroll
    for (int j = 0; j < DX; ++j) {
      if (j < DR && j < nchunks) stage_r(j);
      if (j < nchunks) stage_x(j);
    }
    if (nchunks > DX) wait_vm_at_most<kAllowed>(); else wait_vm_at_most<0>();  // chunk 0 has landed
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
      // ring slots written now were last read in chunk c - 1, whose closing barrier every wave has passed
      if (c + DR < nchunks) stage_r(c + DR);
      const bool more_x = c + DX < nchunks;
      if (!kSpreadX && more_x) stage_x(c + DX);
      const uint4* bufa = lds + (c % (DR + 1)) * S::kSlotsR;
      const uint4* bufb = lds_x + (c % (DX + 1)) * S::kSlotsX;
      uint4 fa[2][MTW], fb[2][NTW];          // fragments of the step in flight and of the next one
#pragma unroll
      for (int t = 0; t < MTW; ++t) fa[0][t] = bufa[a_tile(t) + fslot[0]];
#pragma unroll
      for (int u = 0; u < NTW; ++u) fb[0][u] = bufb[b_tile0 + u * 32 * kPieces + fslot[0]];
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        if (s + 1 < kSteps) {
#pragma unroll
          for (int t = 0; t < MTW; ++t) fa[(s + 1) & 1][t] = bufa[a_tile(t) + fslot[s + 1]];
#pragma unroll
          for (int u = 0; u < NTW; ++u) fb[(s + 1) & 1][u] = bufb[b_tile0 + u * 32 * kPieces + fslot[s + 1]];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < MTW; ++t)
#pragma unroll
          for (int u = 0; u < NTW; ++u) Mma<DT>::run(fa[s & 1][t], fb[s & 1][u], acc[t][u]);
        __builtin_amdgcn_sched_barrier(0);
        if (kSpreadX && more_x) stage_x_part(c + DX, s);   // behind the step's MFMAs, which are queued by now
      }
      // chunk c + 1 must have landed: everything but the loads issued after it (none of them near the end)
      if (c + DX < nchunks) wait_vm_at_most<kAllowed>(); else wait_vm_at_most<0>();
      __syncthreads();
    }

    uint2* ex = reinterpret_cast<uint2*>(lds);   // [HALVES][kTokens][nh]: {magnitude bits, row | sign << 31}
    if constexpr (RC != 0) {
      // r is the constant RC: this wave's MTW tiles are kSeg whole hashes (for r = 256, half of the one hash)
      constexpr int kSegTiles = RC / 32 < MTH ? RC / 32 : MTH;   // tiles per hash inside this wave
      constexpr int kSeg = MTH / kSegTiles;                      // hashes (or hash parts) per wave
      const int mhu = __builtin_amdgcn_readfirstlane(mh);
      static_for<kSeg>([&](auto sc) {
        constexpr int sg = decltype(sc)::value;
        const int lh = RC == 256 ? 0 : mhu * kSeg + sg;          // hash of this segment inside the group (wave-uniform)
        if (lh < nh) {
          float bv[NTW];
          int bid[NTW];
          scan_hash_tiles<sg * kSegTiles, kSegTiles>(acc, bv, bid);
          static_for<NTW>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            int bi = bid[u] + 4 * h + (RC == 256 ? mhu * 128 : 0);
            bool neg;
            const uint32_t best = join_lane_halves(bv[u], bi, neg);
            if (HALVES == 1) {
              b[u] = b[u] * (uint64_t)(2 * RC) + (uint64_t)(bi + (neg ? RC : 0));
            } else if (h == 0) {
              ex[((mh * S::kTokens) + g * NTW * 32 + u * 32 + n) * nh + lh] =
                  make_uint2(best, (uint32_t)bi | (neg ? 0x80000000u : 0u));
            }
          });
        }
      });
    } else {
    // Signed arg-max per hash over the rows this wave holds (tiles mh*MTW .. mh*MTW + MTW-1).  Same two-pass
    // integer scheme as hash_kernel's aligned epilogue.  With two halves the results are joined through LDS.
    for (int lh = 0; lh < nh; ++lh) {
      const int lo = lh * r;
#pragma unroll
      for (int u = 0; u < NTW; ++u) {
        int pmax = (int)0x80000000;
        uint32_t nmax = 0;
#pragma unroll
        for (int t = 0; t < MTH; ++t) {
          const int row0 = (mh * MTH + t) * 32;
          if (row0 + 31 < lo || row0 >= lo + r) continue;  // wave-uniform
#pragma unroll
          for (int jb = 0; jb < 4; ++jb) {
            const int base = row0 + 8 * jb - lo;
            if (base < 0 || base >= r) continue;           // wave-uniform
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const uint32_t vi = __float_as_uint(acc[t][u][4 * jb + i]);
              pmax = max(pmax, (int)vi);
              nmax = max(nmax, vi);
            }
          }
        }
        const uint32_t mp = pmax >= 0 ? (uint32_t)pmax : 0u;
        const uint32_t mn = (nmax >> 31) ? (nmax & 0x7fffffffu) : 0u;
        uint32_t best = max(mp, mn);
        bool neg = mn > mp;
        const float bestf = __uint_as_float(best);
        int bi = 0x7fffffff;
        uint32_t wbits = neg ? 0x80000000u : 0u;           // pattern of the value at the lowest row of largest magnitude
#pragma unroll
        for (int t = MTH - 1; t >= 0; --t) {
          const int row0 = (mh * MTH + t) * 32;
          if (row0 + 31 < lo || row0 >= lo + r) continue;
#pragma unroll
          for (int jb = 3; jb >= 0; --jb) {
            const int base = row0 + 8 * jb - lo;
            if (base < 0 || base >= r) continue;
#pragma unroll
            for (int i = 3; i >= 0; --i) {
              const float v = acc[t][u][4 * jb + i];
              if (fabsf(v) == bestf) {
                bi = base + 4 * h + i;
                wbits = __float_as_uint(v);
              }
            }
          }
        }
        if (mp == mn && best != 0u) neg = (wbits >> 31) != 0u;  // +m and -m both present: the lowest row decides
        // the other 16 rows of each tile sit in lane l ^ 32
        const uint32_t obest = (uint32_t)__shfl_xor((int)best, 32, 64);
        const int obi = __shfl_xor(bi, 32, 64);
        const int oneg = __shfl_xor((int)neg, 32, 64);
        if (obest > best || (obest == best && obi < bi)) {
          best = obest;
          bi = obi;
          neg = oneg != 0;
        }
        if (HALVES == 1) {
          b[u] = b[u] * (uint64_t)(2 * r) + (uint64_t)(bi + (neg ? r : 0));
        } else if (h == 0) {
          ex[((mh * S::kTokens) + g * NTW * 32 + u * 32 + n) * nh + lh] =
              make_uint2(best, (uint32_t)bi | (neg ? 0x80000000u : 0u));
        }
      }
    }
    }
    if (GATE) {
      // rows rows_h .. rows_h + E - 1 are gate logits: a lane holds 4 consecutive ones of its token per register quad
#pragma unroll
      for (int u = 0; u < NTW; ++u) {
        const uint32_t tok = tok_blk + (uint32_t)(g * NTW * 32 + u * 32 + n);
#pragma unroll
        for (int t = GSPLIT ? MTH : 0; t < MTW; ++t) {
#pragma unroll
          for (int jb = 0; jb < 4; ++jb) {
            // rows_h is a multiple of 8: e0 is a multiple of 4.  With two halves the wave's gate tile holds gate rows
            // 32 mh .. 32 mh + 31.
            const int e0 = GSPLIT ? mh * 32 + 8 * jb + 4 * h : t * 32 + 8 * jb + 4 * h - rows_h;
            if (tok >= T || e0 < 0 || e0 >= E) continue;
            float* dst = logits + (size_t)tok * E + e0;
            if (e0 + 3 < E && (E & 3) == 0) {
              *reinterpret_cast<float4*>(dst) = make_float4(acc[t][u][4 * jb], acc[t][u][4 * jb + 1],
                                                            acc[t][u][4 * jb + 2], acc[t][u][4 * jb + 3]);
            } else {
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (e0 + i < E) dst[i] = acc[t][u][4 * jb + i];
            }
          }
        }
      }
    }
    if (HALVES == 2) {
      __syncthreads();                       // both halves of every token are in LDS
      if (mh == 0 && h == 0) {
#pragma unroll
        for (int u = 0; u < NTW; ++u) {
          const int tok = g * NTW * 32 + u * 32 + n;
          for (int lh = 0; lh < nh; ++lh) {
            uint32_t code;
            if constexpr (RC != 0 && RC != 256) {
              // whole hashes per wave: hash lh was finished by the wave of half lh / (hashes per wave)
              constexpr int kPerWave = MTH * 32 / RC;
              code = ex[((lh / kPerWave) * S::kTokens + tok) * nh + lh].y;
            } else {
              const uint2 lo_half = ex[tok * nh + lh], hi_half = ex[(S::kTokens + tok) * nh + lh];
              code = lo_half.y;
              // rows of the upper half are higher, so on equal magnitude the lower half wins unless it holds no row
              if (hi_half.x > lo_half.x || (hi_half.x == lo_half.x && (hi_half.y & 0x7fffffffu) < (code & 0x7fffffffu)))
                code = hi_half.y;
            }
            b[u] = b[u] * (uint64_t)(2 * r) + (uint64_t)((code & 0x7fffffffu) + ((code >> 31) ? (uint32_t)r : 0u));
          }
        }
      }
    }
  }
  if (mh == 0 && h == 0 && (!GATE || L > 0)) {
#pragma unroll
    for (int u = 0; u < NTW; ++u) {
      const uint32_t tok = tok_blk + (uint32_t)(g * NTW * 32 + u * 32 + n);
      if (tok < T) bucket[tok] = b[u];
    }
  }
}

template <typename DT, int MTW, int NTW, int GROUPS, int HALVES, int DR, int DX, bool GATE = false, int RC = 0>
hipError_t launch_stream(const char* x, const char* R, uint64_t* bucket, int64_t T, int row_pieces, int L, int r, int hpg,
                         hipStream_t stream, const char* gate_w = nullptr, int E = 0, float* logits = nullptr) {
  using S = StreamShape<MTW, NTW, GROUPS, HALVES, DR, DX>;
  static_assert(S::kLdsBytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
  if ((GATE ? L * r + E : hpg * r) > S::kRows) return hipErrorInvalidValue;  // the instance must hold every row of a pass
  if (GATE && HALVES == 2 && (L * r > HALVES * (MTW - 1) * 32 || E > HALVES * 32 || L < 1)) return hipErrorInvalidValue;
  if (RC != 0 && r != RC) return hipErrorInvalidValue;                       // a compile-time r must be the real one
  auto kern = hash_stream_kernel<DT, MTW, NTW, GROUPS, HALVES, DR, DX, GATE, RC>;
  static std::atomic<bool> raised{false};  // set once per kernel; repeating the call is harmless
  if (!raised.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::kLdsBytes);
    if (e != hipSuccess) return e;
    raised.store(true, std::memory_order_release);
  }
  const dim3 grid((uint32_t)((T + S::kTokens - 1) / S::kTokens)), block(S::kWaves * 64);
  hipLaunchKernelGGL(kern, grid, block, S::kLdsBytes, stream, x, R, bucket, (uint32_t)T, row_pieces, L, r, hpg, gate_w, E,
                     logits);
  return hipGetLastError();
}

template <typename DT, int MT, int NTK, int XDEPTH, int WAVES, int OCC, bool ALIGNED8, bool KTAIL>
hipError_t launch_one(const char* x, const char* R, uint64_t* bucket, int64_t T, int row_pieces, int L, int r, int hpg,
                      hipStream_t stream) {
  constexpr int kBlockTokens = WAVES * NTK * 32;
  if (hpg < 1 || hpg * r > MT * 32) return hipErrorInvalidValue;  // the instance must hold every row of a pass
  constexpr size_t lds_bytes = (size_t)2 * MT * 32 * kPieces * 16;
  static_assert(lds_bytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
  auto kern = hash_kernel<DT, MT, NTK, XDEPTH, WAVES, OCC, ALIGNED8, KTAIL>;
  if (lds_bytes > 48 * 1024) {
    static std::atomic<bool> raised{false};  // set once per kernel; repeating the call is harmless
    if (!raised.load(std::memory_order_acquire)) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
      if (e != hipSuccess) return e;
      raised.store(true, std::memory_order_release);
    }
  }
  const dim3 grid((uint32_t)((T + kBlockTokens - 1) / kBlockTokens)), block(WAVES * 64);
  hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, x, R, bucket, (uint32_t)T, row_pieces, L, r, hpg,
                     (const float*)nullptr);
  return hipGetLastError();
}

template <typename DT>
hipError_t launch_typed(const void* tokens, const void* rot, int64_t T, int d, int L, int r, uint64_t* bucket,
                        hipStream_t stream) {
  int hpg = 256 / r;                       // whole hashes per pass over the tokens
  if (hpg > L) hpg = L;
  if (hpg < 1) return hipErrorInvalidValue;
  const int mt = (hpg * r + 31) / 32;
  const int row_pieces = (int)((size_t)d * ItemSize<DT>::value / 16);
  auto x = (const char*)tokens;
  auto R = (const char*)rot;
  // fast instance: r a multiple of 8 (uniform epilogue) and rows a whole number of 4 x 128-byte chunks (no k tail)
  const bool fast = r % 8 == 0 && row_pieces % (kPieces * 4) == 0;
#define LSHMOE_HASH(MT, NTK, XD, WAVES, OCC)                                                                      \
  (fast ? launch_one<DT, MT, NTK, XD, WAVES, OCC, true, false>(x, R, bucket, T, row_pieces, L, r, hpg, stream)    \
        : launch_one<DT, MT, NTK, XD, WAVES, OCC, false, true>(x, R, bucket, T, row_pieces, L, r, hpg, stream))
  // Workgroup size.  Few rows of R: the kernel is bound by streaming the tokens, so the workgroups are made
  // small enough that at least 512 of them exist (2 per compute unit).  Many rows of R (mt >= 6): the LDS
  // staging of R dominates, and 8 waves sharing one staged copy beat two 4-wave workgroups with one each.
  // OCC: waves per SIMD the register budget is cut for - while one wave waits at a chunk barrier another
  // issues MFMAs.
  // Widest groups on large inputs: the 4 x 2 tiling with the rows of R split between two waves (see hash_stream_kernel).
  // Measured at T = 65536, d = 1024, 256 rows: 42 us against 45 us with tokens coming from HBM, 47 us against
  // 43 us when the tokens are still in the last-level cache.
  if (mt >= 7 && fast && T >= 256 * 256) {
#define LSHMOE_WIDE(RC) launch_stream<DT, 4, 2, 4, 2, 1, 2, false, RC>(x, R, bucket, T, row_pieces, L, r, hpg, stream)
    return r == 64 ? LSHMOE_WIDE(64) : r == 128 ? LSHMOE_WIDE(128) : r == 256 ? LSHMOE_WIDE(256)
         : r == 32 ? LSHMOE_WIDE(32) : LSHMOE_WIDE(0);
#undef LSHMOE_WIDE
  }
  // Few rows of R (mt <= 4): the kernel is bound by streaming the tokens.  From about 8k tokens on the streaming
  // kernel wins (measured per call: GPT shape 23.7 -> 18.9 us, Swin 12.7 -> 10.6, RoBERTa 13.1 -> 10.7): 128-token
  // workgroups of four waves with the tokens four chunks ahead once there are enough tokens for ~200 of them,
  // else 64-token workgroups of two waves three chunks ahead.
  if (fast && mt <= 4 && T >= 8192) {
    const bool big = T >= 24576;
    // beyond 256 workgroups of 128 tokens (one per compute unit): shorter rings (at most 80 KB), so that two
    // workgroups share a compute unit's LDS and the workgroups past the first 256 do not wait for a second round
    // (measured at T = 65536, d = 1024: 64 rows 29.8 -> 26.8 us, 128 rows 34.1 -> 29.3 us; T = 131072, 128 rows 65.8 -> 54.5 us)
    const bool huge = T > 256 * 128;
#define LSHMOE_STREAM(MT, RC) \
    (huge ? launch_stream<DT, MT, 1, 4, 1, 1, 2, false, RC>(x, R, bucket, T, row_pieces, L, r, hpg, stream) \
     : big ? launch_stream<DT, MT, 1, 4, 1, 3, 4, false, RC>(x, R, bucket, T, row_pieces, L, r, hpg, stream) \
           : launch_stream<DT, MT, 1, 2, 1, 2, 3, false, RC>(x, R, bucket, T, row_pieces, L, r, hpg, stream))
    // r = 32 and r = 64 (whole hashes per tile or per two tiles) take the arg-max with compile-time row ranges
    if (mt <= 1) return r == 32 ? LSHMOE_STREAM(1, 32) : LSHMOE_STREAM(1, 0);
    if (mt == 2) return r == 32 ? LSHMOE_STREAM(2, 32) : r == 64 ? LSHMOE_STREAM(2, 64) : LSHMOE_STREAM(2, 0);
    if (mt == 3) return r == 32 ? LSHMOE_STREAM(3, 32) : LSHMOE_STREAM(3, 0);
    return r == 32 ? LSHMOE_STREAM(4, 32) : r == 64 ? LSHMOE_STREAM(4, 64) : LSHMOE_STREAM(4, 0);
#undef LSHMOE_STREAM
  }
  if (mt >= 5) {                           // 129..192 rows take the 6-tile instance, more the 8-tile one
    const bool wide = T >= 256 * 256;
    if (mt <= 6) return wide ? LSHMOE_HASH(6, 1, 2, 8, 1) : LSHMOE_HASH(6, 1, 2, 4, 2);
    return wide ? LSHMOE_HASH(8, 1, 2, 8, 1) : LSHMOE_HASH(8, 1, 2, 4, 2);
  }
  const int waves = T >= 512 * 128 ? 4 : T >= 512 * 64 ? 2 : 1;
#define LSHMOE_HASH_SMALL(MT)                                       \
  (waves == 4 ? LSHMOE_HASH(MT, 1, 4, 4, 2) : waves == 2 ? LSHMOE_HASH(MT, 1, 4, 2, 2) : LSHMOE_HASH(MT, 1, 4, 1, 2))
  if (mt <= 1) return LSHMOE_HASH_SMALL(1);
  if (mt == 2) return LSHMOE_HASH_SMALL(2);
  if (mt == 3) return LSHMOE_HASH_SMALL(3);
  return LSHMOE_HASH_SMALL(4);
#undef LSHMOE_HASH_SMALL
#undef LSHMOE_HASH
}

// Spherical hash: B spheres (rows of `pivots`), one or two 32-row tiles, tokens straight into registers.
template <typename DT>
hipError_t launch_sphere_typed(const void* tokens, const void* pivots, const float* radius_sq, int64_t T, int d, int B,
                               uint64_t* bucket, hipStream_t stream) {
  if (B < 1 || B > 63) return hipErrorInvalidValue;
  const int row_pieces = (int)((size_t)d * ItemSize<DT>::value / 16);
  constexpr int kWaves = 4, kBlockTokens = kWaves * 32;
  const dim3 grid((uint32_t)((T + kBlockTokens - 1) / kBlockTokens)), block(kWaves * 64);
  if (B <= 32) {
    constexpr size_t lds_bytes = (size_t)2 * 32 * kPieces * 16;
    hipLaunchKernelGGL((hash_kernel<DT, 1, 1, 4, kWaves, 2, false, true, true>), grid, block, lds_bytes, stream,
                       (const char*)tokens, (const char*)pivots, bucket, (uint32_t)T, row_pieces, 1, B, 1, radius_sq);
  } else {
    constexpr size_t lds_bytes = (size_t)2 * 64 * kPieces * 16;
    hipLaunchKernelGGL((hash_kernel<DT, 2, 1, 4, kWaves, 2, false, true, true>), grid, block, lds_bytes, stream,
                       (const char*)tokens, (const char*)pivots, bucket, (uint32_t)T, row_pieces, 1, B, 1, radius_sq);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_hash_sphere(const void* tokens, const void* pivots, const float* radius_sq, int64_t T, int d, int B,
                              bool bf16, uint64_t* bucket, hipStream_t stream) {
  return bf16 ? launch_sphere_typed<BF16>(tokens, pivots, radius_sq, T, d, B, bucket, stream)
              : launch_sphere_typed<F32>(tokens, pivots, radius_sq, T, d, B, bucket, stream);
}

namespace {

// Gate rows (and, when they fit, the hash rows in front of them) on the streaming kernel: mt row tiles per wave.
template <typename DT>
hipError_t launch_gate_rows(const char* x, const char* R, const char* W, int64_t T, int row_pieces, int L, int r, int E,
                            uint64_t* bucket, float* logits, hipStream_t stream) {
  const int mt = (L * r + E + 31) / 32;
  const bool big = T >= 24576;
  const bool huge = T > 256 * 128;   // as for the hash alone: two workgroups per compute unit
#define LSHMOE_GATE(MT)                                                                                               \
  (huge ? launch_stream<DT, MT, 1, 4, 1, 1, 2, true>(x, R, bucket, T, row_pieces, L, r, L > 0 ? L : 1, stream, W, E, logits) \
   : big ? launch_stream<DT, MT, 1, 4, 1, 3, 4, true>(x, R, bucket, T, row_pieces, L, r, L > 0 ? L : 1, stream, W, E, logits) \
         : launch_stream<DT, MT, 1, 2, 1, 2, 3, true>(x, R, bucket, T, row_pieces, L, r, L > 0 ? L : 1, stream, W, E, logits))
  if (mt <= 1) return LSHMOE_GATE(1);
  if (mt == 2) return LSHMOE_GATE(2);
  if (mt == 3) return LSHMOE_GATE(3);
  return LSHMOE_GATE(4);
#undef LSHMOE_GATE
}

template <typename DT>
hipError_t launch_hash_gate_typed(const void* tokens, const void* rot, const void* gate_w, int64_t T, int d, int L, int r,
                                  int E, uint64_t* bucket, float* logits, hipStream_t stream) {
  const int row_pieces = (int)((size_t)d * ItemSize<DT>::value / 16);
  auto x = (const char*)tokens;
  auto R = (const char*)rot;
  auto W = (const char*)gate_w;
  if ((int64_t)L * r + E <= 128)  // one pass over the tokens for both
    return launch_gate_rows<DT>(x, R, W, T, row_pieces, L, r, E, bucket, logits, stream);
  // Up to 256 rows of R and 64 gate rows on large inputs: still one pass, on the shape of the widest hash instance
  // with a fifth tile per wave for the gate rows.  All of LDS goes to two ring slots per operand, so the tokens run
  // only one chunk ahead; that is slower per chunk than the hash alone but far cheaper than a second pass over the
  // tokens (measured at T = 65536, d = 1024, 256 + 64 rows: see the benchmark's supplementary_hash_gate).
  if ((int64_t)L * r <= 256 && E <= 64 && T >= 32768) {
#define LSHMOE_GATE_WIDE(RC) launch_stream<DT, 5, 2, 4, 2, 1, 1, true, RC>(x, R, bucket, T, row_pieces, L, r, L, stream, W, E, logits)
    return r == 64 ? LSHMOE_GATE_WIDE(64) : r == 32 ? LSHMOE_GATE_WIDE(32) : r == 128 ? LSHMOE_GATE_WIDE(128) : LSHMOE_GATE_WIDE(0);
#undef LSHMOE_GATE_WIDE
  }
  // too many rows for one accumulator set: the hash as usual, then the gate rows alone (the tokens are read twice)
  hipError_t e = launch_typed<DT>(tokens, rot, T, d, L, r, bucket, stream);
  if (e != hipSuccess) return e;
  return launch_gate_rows<DT>(x, R, W, T, row_pieces, 0, r, E, bucket, logits, stream);
}

}  // namespace

bool hash_gate_supported(int d, int r, int E, bool bf16) {
  const int row_pieces = (int)((size_t)d * (bf16 ? 2 : 4) / 16);
  return r % 8 == 0 && row_pieces % (kPieces * 4) == 0 && E >= 1 && E <= 128;
}

hipError_t launch_hash_gate(const void* tokens, const void* rot, const void* gate_w, int64_t T, int d, int L, int r, int E,
                            bool bf16, uint64_t* bucket, float* logits, hipStream_t stream) {
  return bf16 ? launch_hash_gate_typed<BF16>(tokens, rot, gate_w, T, d, L, r, E, bucket, logits, stream)
              : launch_hash_gate_typed<F32>(tokens, rot, gate_w, T, d, L, r, E, bucket, logits, stream);
}

hipError_t launch_hash(const void* tokens, const void* rot, int64_t T, int d, int L, int r, bool bf16,
                       uint64_t* bucket, hipStream_t stream) {
  return bf16 ? launch_typed<BF16>(tokens, rot, T, d, L, r, bucket, stream)
              : launch_typed<F32>(tokens, rot, T, d, L, r, bucket, stream);
}

}  // namespace lshmoe
