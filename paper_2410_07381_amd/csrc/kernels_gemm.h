// bf16 GEMM logical-block body for gfx950: one 256x256 output tile per logical block.
//
// C = A * B with A (m x k) and Bt (n x k) both K-contiguous, so an MFMA operand fragment
// (8 consecutive bf16 along K) is one 16-byte access for either matrix.  Four 64-lane
// waves in a 2x2 arrangement each own a 128x128 sub-tile as 4x4 MFMA 32x32x16 blocks
// (256 fp32 accumulators per lane, which the compiler keeps in accumulation registers).
// K is walked in steps of 64 through two LDS buffers per operand (128 KB in all).
//
// Global memory goes straight to LDS (16 bytes per lane, no staging registers): a wave
// load fills 1 KB of LDS contiguously, lane l supplying the 16-byte slot l.  Slot s of a
// tile holds row s/8, k-chunk (s%8) xor (row%8); the xor makes the 8 lanes that an LDS
// read serves together fall into 8 different 16-byte bank groups, without padding.  The
// lane-to-address map of the global side is chosen to produce that layout; it still
// reads whole 128-byte row segments.
//
// Register budget: the arithmetic VGPRs are kept low on purpose so that, with the 256
// accumulators, a wave stays well under the 512 registers of its SIMD and waves of a
// high-priority kernel can become resident beside a running tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tally.h"
#include "kernels_stream.h"

namespace tally {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

struct GemmBody {
  using Args = tally_gemm_bf16_args;
  static constexpr int THREADS = 256;
  static constexpr int MIN_WAVES = 1;
  static constexpr int TILE = 256;
  static constexpr int BK = 64;
  static constexpr int BUF = TILE * BK;                   // one operand buffer, in bf16 (32 KB)
  static constexpr unsigned DYN_LDS = 4u * BUF * 2u;      // A0 A1 B0 B1 = 128 KB
  // every k-step ends with a barrier after its LDS reads, so the next tile's first loads
  // cannot overtake a reader of this tile
  static constexpr bool END_BARRIER = false;

  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t by, uint32_t bz) {
    extern __shared__ __align__(1024) unsigned char tally_dyn_lds[];
    unsigned char *sA = tally_dyn_lds;
    unsigned char *sB = tally_dyn_lds + 2 * BUF * 2;

    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
    const uint32_t K = a.k;

    // global side of the direct loads: wave w fills rows [64 w, 64 w + 64) of each operand
    // tile with 8 loads of 8 rows; lane l supplies row l/8, k-chunk (l%8) xor (l/8)
    const uint32_t ld_row = wave * 64 + (lane >> 3);
    const uint32_t ld_kc = (lane & 7) ^ (lane >> 3);
    const uint16_t *pA = a.A + bz * a.stride_a + (uint64_t)(by * TILE + ld_row) * K + ld_kc * 8;
    const uint16_t *pB = a.Bt + bz * a.stride_b + (uint64_t)(bx * TILE + ld_row) * K + ld_kc * 8;
    const uint32_t lds_wave = wave * 64 * BK * 2;           // byte offset of the wave's rows

    auto issue_loads = [&](uint32_t kt, uint32_t buf) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        __builtin_amdgcn_global_load_lds((gptr_t)(pA + (uint64_t)(8 * j) * K + kt * BK),
                                         (lptr_t)(sA + buf * BUF * 2 + lds_wave + j * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gptr_t)(pB + (uint64_t)(8 * j) * K + kt * BK),
                                         (lptr_t)(sB + buf * BUF * 2 + lds_wave + j * 1024), 16, 0, 0);
      }
    };

    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const uint32_t nk = K / BK;
    issue_loads(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // fragment reads: lane l takes row (l%32) of a 32-row block and k-chunk 2 ks + l/32;
    // (row % 8) == (l % 8) because every 32-row block starts on a multiple of 8
    const uint32_t f_row = lane & 31, f_half = lane >> 5, f_x = lane & 7;
    const uint32_t fA = (wm * 128 + f_row) * (BK * 2);
    const uint32_t fB = (wn * 128 + f_row) * (BK * 2);
    for (uint32_t kt = 0; kt < nk; ++kt) {
      const uint32_t buf = kt & 1;
      if (kt + 1 < nk) issue_loads(kt + 1, buf ^ 1);
      const unsigned char *cA = sA + buf * BUF * 2 + fA;
      const unsigned char *cB = sB + buf * BUF * 2 + fB;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        const uint32_t koff = ((uint32_t)(2 * ks + f_half) ^ f_x) * 16;
        bf16x8_t fa[4], fb[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          fa[t] = *reinterpret_cast<const bf16x8_t *>(cA + t * 32 * BK * 2 + koff);
          fb[t] = *reinterpret_cast<const bf16x8_t *>(cB + t * 32 * BK * 2 + koff);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
      // the other buffer must be completely written, and this one completely read,
      // before the next step swaps them
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          uint32_t row = row0 + i * 32 + (r >> 2) * 8 + (r & 3);
          uint32_t col = col0 + j * 32;
          // read each accumulator where it is used: a wholesale copy of the 256
          // accumulators into arithmetic registers would double the wave's register
          // footprint, which decides how many other waves fit beside this one
          float v;
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][r]));
          gC[(uint64_t)row * a.n + col] = f32_to_bf16(v);
        }
      }
  }
};

// Same operator with 64x64 output tiles and predicated edges, for small or ragged
// problems (the high-priority inference-like layer).  One wave per 32x32 block.
struct GemmSmallBody {
  using Args = tally_gemm_bf16_args;
  static constexpr int THREADS = 256;
  static constexpr int MIN_WAVES = 2;
  static constexpr int TILE = 64;
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool END_BARRIER = false;

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
