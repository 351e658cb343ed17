// bf16 GEMM logical-block body for gfx950: one 256x256 output tile per logical block.
//
// C = A * B with A (m x k) and Bt (n x k) both K-contiguous, so an MFMA operand fragment
// (8 consecutive bf16 along K) is one 16-byte access for either matrix.  Four 64-lane
// waves in a 2x2 arrangement each own a 128x128 sub-tile as 4x4 MFMA 32x32x16 blocks
// (256 fp32 accumulators per lane).  K is walked in steps of 64 through two LDS buffers
// per operand; rows are padded to 72 bf16 (144 B) so the 16 lanes served together by a
// 128-bit LDS read fall in distinct bank groups.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tally.h"
#include "kernels_stream.h"

namespace tally {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

struct GemmBody {
  using Args = tally_gemm_bf16_args;
  static constexpr int THREADS = 256;
  static constexpr int TILE = 256;
  static constexpr int BK = 64;
  static constexpr int LDK = 72;                          // padded LDS row, in bf16
  static constexpr int BUF = TILE * LDK;                  // one operand buffer, in bf16
  static constexpr unsigned DYN_LDS = 4u * BUF * 2u;      // A0 A1 B0 B1

  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t by, uint32_t bz) {
    extern __shared__ __align__(16) unsigned char tally_dyn_lds[];
    uint16_t *sA = reinterpret_cast<uint16_t *>(tally_dyn_lds);
    uint16_t *sB = sA + 2 * BUF;

    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
    const uint32_t K = a.k;
    const uint16_t *gA = a.A + bz * a.stride_a + (uint64_t)(by * TILE) * K;
    const uint16_t *gB = a.Bt + bz * a.stride_b + (uint64_t)(bx * TILE) * K;

    // global -> LDS mapping: 16-byte chunk c = tid + 256 j covers row c/8, k-chunk c%8
    const uint32_t ld_row = tid >> 3, ld_kc = tid & 7;      // + 32 rows per j
    const uint16_t *pA = gA + (uint64_t)ld_row * K + ld_kc * 8;
    const uint16_t *pB = gB + (uint64_t)ld_row * K + ld_kc * 8;
    const uint32_t st_off = ld_row * LDK + ld_kc * 8;       // + 32 * LDK per j

    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 ra[8], rb[8];
    auto gload = [&](uint32_t kt) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        ra[j] = *reinterpret_cast<const uint4 *>(pA + (uint64_t)(32 * j) * K + kt * BK);
        rb[j] = *reinterpret_cast<const uint4 *>(pB + (uint64_t)(32 * j) * K + kt * BK);
      }
    };
    auto lstore = [&](uint32_t buf) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        *reinterpret_cast<uint4 *>(sA + buf * BUF + st_off + 32 * j * LDK) = ra[j];
        *reinterpret_cast<uint4 *>(sB + buf * BUF + st_off + 32 * j * LDK) = rb[j];
      }
    };

    const uint32_t nk = K / BK;
    gload(0);
    lstore(0);
    __syncthreads();

    // fragment addresses: lane l reads row (l & 31) of a 32-row block, k offset 8 (l >> 5)
    const uint32_t fr = (lane & 31) * LDK + (lane >> 5) * 8;
    for (uint32_t kt = 0; kt < nk; ++kt) {
      const uint32_t buf = kt & 1;
      if (kt + 1 < nk) gload(kt + 1);
      const uint16_t *cA = sA + buf * BUF + (wm * 128) * LDK + fr;
      const uint16_t *cB = sB + buf * BUF + (wn * 128) * LDK + fr;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8_t fa[4], fb[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          fa[t] = *reinterpret_cast<const bf16x8_t *>(cA + t * 32 * LDK + ks * 16);
          fb[t] = *reinterpret_cast<const bf16x8_t *>(cB + t * 32 * LDK + ks * 16);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
      if (kt + 1 < nk) lstore(buf ^ 1);
      __syncthreads();
    }

    // epilogue: lane l, register r of a 32x32 block holds row 8 (r/4) + 4 (l/32) + r%4,
    // column l%32
    uint16_t *gC = a.C + bz * a.stride_c;
    const uint32_t row0 = by * TILE + wm * 128 + (lane >> 5) * 4;
    const uint32_t col0 = bx * TILE + wn * 128 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          uint32_t row = row0 + i * 32 + (r >> 2) * 8 + (r & 3);
          uint32_t col = col0 + j * 32;
          gC[(uint64_t)row * a.n + col] = f32_to_bf16(acc[i][j][r]);
        }
  }
};

// Same operator with 64x64 output tiles and predicated edges, for small or ragged
// problems (the high-priority inference-like layer).  One wave per 32x32 block.
struct GemmSmallBody {
  using Args = tally_gemm_bf16_args;
  static constexpr int THREADS = 256;
  static constexpr int TILE = 64;
  static constexpr unsigned DYN_LDS = 0;

  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t by, uint32_t bz) {
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
    const uint32_t K = a.k;
    const uint32_t arow = by * TILE + wm * 32 + (lane & 31);
    const uint32_t brow = bx * TILE + wn * 32 + (lane & 31);
    const bool aok = arow < a.m, bok = brow < a.n;
    const uint16_t *pA = a.A + bz * a.stride_a + (uint64_t)(aok ? arow : 0) * K + (lane >> 5) * 8;
    const uint16_t *pB = a.Bt + bz * a.stride_b + (uint64_t)(bok ? brow : 0) * K + (lane >> 5) * 8;
    f32x16_t acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
    const uint4 zero = make_uint4(0, 0, 0, 0);
    // operands straight from global/L2: each 16-byte fragment is used by this wave only
    // once per k step, and the 2x2 waves of a block share rows through the L1
    for (uint32_t k0 = 0; k0 < K; k0 += 32) {
      uint4 a0 = aok ? *reinterpret_cast<const uint4 *>(pA + k0) : zero;
      uint4 b0 = bok ? *reinterpret_cast<const uint4 *>(pB + k0) : zero;
      uint4 a1 = aok ? *reinterpret_cast<const uint4 *>(pA + k0 + 16) : zero;
      uint4 b1 = bok ? *reinterpret_cast<const uint4 *>(pB + k0 + 16) : zero;
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a0),
                                                     __builtin_bit_cast(bf16x8_t, b0), acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a1),
                                                     __builtin_bit_cast(bf16x8_t, b1), acc1, 0, 0, 0);
    }
    uint16_t *gC = a.C + bz * a.stride_c;
    const uint32_t col = bx * TILE + wn * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      uint32_t row = by * TILE + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
      if (row < a.m && col < a.n) gC[(uint64_t)row * a.n + col] = f32_to_bf16(acc0[r] + acc1[r]);
    }
  }
};

}  // namespace tally
