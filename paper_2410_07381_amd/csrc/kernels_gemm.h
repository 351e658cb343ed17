// bf16 GEMM logical-block body for gfx950: one 256x256 (or 256x128) output tile per logical
// block.
//
// C = A * B with A (m x k) and Bt (n x k) both K-contiguous, so an MFMA operand fragment
// (8 consecutive bf16 along K) is one 16-byte access for either matrix.  Four 64-lane
// waves in a 2x2 arrangement each own a 128x128 sub-tile as 4x4 MFMA 32x32x16 blocks
// (256 fp32 accumulators per lane, which stay in accumulation registers).
//
// K is walked in steps of 32 through a ring of FOUR LDS stages (32 KB each, 128 KB in
// all): the loads of step i+3 are issued while step i is multiplied, so a tile tolerates
// about three step-times of memory latency.  With two stages of 64 the kernel spent more
// than half its time waiting for the next stage (L2/Infinity-Cache latency under load is
// longer than one step of MFMA work).
//
// Global memory goes straight to LDS (16 bytes per lane, no staging registers): a wave
// load fills 1 KB of LDS contiguously, lane l supplying the 16-byte slot l.  A stage
// holds 256 rows of 64 bytes; slot s holds row s/4, k-chunk (s%4) xor ((row/4)%4), which
// makes the 16 lanes that a 128-bit LDS read serves together (64 banks, 256 bytes per
// clock) fall into 16 different 16-byte bank groups, without padding; with the xor taken
// from row/2 the bank-conflict counter showed every read served at half rate.  The
// lane-to-address map of the global side is chosen to produce that layout.
//
// Register budget: the arithmetic VGPRs are kept low on purpose so that, with the 256
// accumulators, a wave stays well under the 512 registers of its SIMD and waves of a
// high-priority kernel can become resident beside a running tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tally.h"
#include "kernels_stream.h"
#include "launch_forms.h"

namespace tally {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// NB = 32-column MFMA blocks per wave: 4 gives the 256x256 tile, 2 a 256x128 tile (128
// accumulators per lane) for operands whose n is only a multiple of 128.
template <int NB>
struct GemmBodyT {
  static_assert(NB == 2 || NB == 4, "two or four column blocks per wave");
  using Args = tally_gemm_bf16_args;
  static constexpr int THREADS = 256;
  static constexpr int MIN_WAVES = 1;
  static constexpr int TILE = 256;                        // rows of C per logical block
  static constexpr int TILE_N = 64 * NB;                  // columns of C per logical block
  static constexpr int BK = 32;
  static constexpr int STAGES = 4;
  static constexpr int OPA = TILE * BK * 2;               // bytes of A in one stage (16 KB)
  static constexpr int OPB = TILE_N * BK * 2;             // bytes of B in one stage
  static constexpr unsigned DYN_LDS = (unsigned)(OPA + OPB) * STAGES;  // 128 KB / 96 KB
  // every k-step starts with a barrier that follows the LDS reads of the step before, so
  // the next tile's first loads cannot overtake a reader of this tile
  static constexpr bool END_BARRIER = false;
  static constexpr bool YIELDS = true;
  static constexpr bool RANGE = false;
  // share of a tile between two looks at the pause word, `every` k-steps apart (host side,
  // for turnaround estimates)
  static double pause_fraction(const Args &a, uint32_t every) {
    const uint32_t nk = a.k / BK;
    return nk > every ? (double)every / nk : 1.0;
  }

  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t by, uint32_t bz) {
    run_impl<false>(a, bx, by, bz, YieldCtl{nullptr, 0, 0, 15});
  }
  // best-effort forms: the output tile is written with non-temporal stores (it is not read
  // again by this kernel and would only push other data out of the caches)
  static __device__ __forceinline__ void run_be(const Args &a, uint32_t bx, uint32_t by, uint32_t bz) {
    run_impl<true>(a, bx, by, bz, YieldCtl{nullptr, 0, 0, 15});
  }
  static __device__ __forceinline__ void run_yielding(const Args &a, uint32_t bx, uint32_t by,
                                                      uint32_t bz, const YieldCtl ctl) {
    run_impl<true>(a, bx, by, bz, ctl);
  }

  template <bool NT>
  static __device__ __forceinline__ void run_impl(const Args &a, uint32_t bx, uint32_t by,
                                                  uint32_t bz, const YieldCtl ctl) {
    extern __shared__ __align__(1024) unsigned char tally_dyn_lds[];
    unsigned char *sA = tally_dyn_lds;                    // STAGES x 16 KB
    unsigned char *sB = tally_dyn_lds + STAGES * OPA;

    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wm = wave >> 1, wn = wave & 1;
    const uint32_t K = a.k;
    const uint32_t LDA = a.lda ? a.lda : K, LDB = a.ldb ? a.ldb : K;   // row pitches

    // global side of the direct loads: wave w fills rows [64 w, 64 w + 64) of A with 4 loads
    // of 16 rows and rows [16 NB w, 16 NB (w + 1)) of B with NB loads; lane l supplies row
    // l/4, k-chunk (l%4) xor ((l/16)%4).  Addresses are split into a wave-uniform base that
    // advances by 64 bytes per k-step and per-lane byte offsets that never change.  The
    // loads of an operand share one LDS base (M0) and differ by the instruction's immediate
    // offset, which also moves the global address; the uniform bases compensate for that.
    const uint32_t ld_kc = (lane & 3) ^ ((lane >> 4) & 3);
    const unsigned char *uA =
        reinterpret_cast<const unsigned char *>(a.A + bz * a.stride_a + (uint64_t)(by * TILE) * LDA);
    const unsigned char *uB =
        reinterpret_cast<const unsigned char *>(a.Bt + bz * a.stride_b + (uint64_t)(bx * TILE_N) * LDB);
    // one per-lane offset per operand; what distinguishes the loads of an operand (16 rows
    // further down, less the 1024 bytes the immediate adds) is uniform and goes to the base
    const uint32_t voffA = ((wave * 64 + (lane >> 2)) * LDA + ld_kc * 8) * 2;
    const uint32_t voffB = ((wave * 16 * NB + (lane >> 2)) * LDB + ld_kc * 8) * 2;
    const uint64_t stepA = (uint64_t)32 * LDA - 1024, stepB = (uint64_t)32 * LDB - 1024;
    const uint32_t ldsA_wave = wave * 64 * BK * 2;        // byte offset of the wave's rows
    const uint32_t ldsB_wave = wave * 16 * NB * BK * 2;

    // one direct load: 16 rows of A (B) of the 64 (16 NB) a wave contributes to a stage
    // (the operands keep ordinary loads in every form: tiles share them through the L2s and
    // the Infinity Cache; with non-temporal loads of both operands a co-located decode step
    // ran as fast as alone, but the GEMM itself took 1.7 to 2.1 times as long, and with
    // non-temporal loads of A alone 1.1 to 1.4 times for a tenth off the decode step)
    constexpr int AUX = 0;
    constexpr int AUXA = 0;
    auto load_a = [&](const unsigned char *g, lptr_t l, int j) {
      if (j == 0) __builtin_amdgcn_global_load_lds((gptr_t)(g + voffA), l, 16, 0, AUXA);
      if (j == 1) __builtin_amdgcn_global_load_lds((gptr_t)(g + stepA + voffA), l, 16, 1024, AUXA);
      if (j == 2) __builtin_amdgcn_global_load_lds((gptr_t)(g + 2 * stepA + voffA), l, 16, 2048, AUXA);
      if (j == 3) __builtin_amdgcn_global_load_lds((gptr_t)(g + 3 * stepA + voffA), l, 16, 3072, AUXA);
    };
    auto load_b = [&](const unsigned char *g, lptr_t l, int j) {
      if (j == 0) __builtin_amdgcn_global_load_lds((gptr_t)(g + voffB), l, 16, 0, AUX);
      if (j == 1) __builtin_amdgcn_global_load_lds((gptr_t)(g + stepB + voffB), l, 16, 1024, AUX);
      if constexpr (NB > 2) {
        if (j == 2) __builtin_amdgcn_global_load_lds((gptr_t)(g + 2 * stepB + voffB), l, 16, 2048, AUX);
        if (j == 3) __builtin_amdgcn_global_load_lds((gptr_t)(g + 3 * stepB + voffB), l, 16, 3072, AUX);
      }
    };
    auto issue_loads = [&](uint32_t kt) {
      const uint32_t st = kt & (STAGES - 1);
      const unsigned char *gA = uA + (uint64_t)kt * (BK * 2);
      const unsigned char *gB = uB + (uint64_t)kt * (BK * 2);
      lptr_t lA = (lptr_t)(sA + st * OPA + ldsA_wave);
      lptr_t lB = (lptr_t)(sB + st * OPB + ldsB_wave);
#pragma unroll
      for (int j = 0; j < 4; ++j) load_a(gA, lA, j);
#pragma unroll
      for (int j = 0; j < NB; ++j) load_b(gB, lB, j);
    };
    constexpr int LOADS = 4 + NB;                         // direct loads per wave per k-step

    f32x16_t acc[4][NB];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const uint32_t nk = K / BK;
    uint32_t pause_left = ctl.ticks;   // what is left of this block's pause budget
    // A tile's first loads (every resident tile starts at once after a launch) and its
    // epilogue (32 MiB written by all compute units together) are its heaviest bursts of
    // memory traffic: a tile long enough to afford two more looks at the pause word takes
    // them just before either, so that neither burst starts on top of a high-priority kernel.
    const bool edge_polls = ctl.ticks != 0 && nk >= 32;
    if (edge_polls && wave == 0) yield_while_preempted(ctl, pause_left);
    // a previous tile's waves may still be reading its last stage: fence them off before
    // refilling the ring
    __syncthreads();
    issue_loads(0);
    if (nk > 1) issue_loads(1);
    if (nk > 2) issue_loads(2);

    // fragment reads: lane l takes row (l%32) of a 32-row block and k-chunk 2 ks + l/32
    const uint32_t f_row = lane & 31, f_half = lane >> 5, f_x = (lane >> 2) & 3;
    const uint32_t fA = (wm * 128 + f_row) * (BK * 2);
    const uint32_t fB = (wn * 32 * NB + f_row) * (BK * 2);
    const uint32_t koff0 = ((0u + f_half) ^ f_x) * 16, koff1 = ((2u + f_half) ^ f_x) * 16;

    // Two fragment sets: the LDS reads of the next half-step travel while the MFMAs of the
    // current one run.  A wave is alone on its SIMD, so whatever it issues between two
    // MFMAs that does not fit into the 32 cycles the earlier MFMA occupies the matrix pipe
    // leaves the pipe idle.  Reads and direct loads are therefore written, and pinned by
    // scheduling groups, one at a time between MFMAs: the reads the first MFMAs of the next
    // half need come first, then the remaining reads alternate with the half's direct
    // loads (with four column blocks three MFMAs apart: the four waves issue theirs
    // together and the address unit takes 16 cycles per 1 KB load).  Reads and direct loads
    // both touch LDS, so the compiler keeps them in source order: the source order below is
    // the issue order.  Against reads and loads bunched in front of sixteen MFMAs this took
    // a quarter of the cycles out of the loop.
    bf16x8_t fa0[4], fb0[NB], fa1[4], fb1[NB];
    auto lfrag = [&](bf16x8_t(&fa)[4], bf16x8_t(&fb)[NB], uint32_t kt, uint32_t koff) {
      const unsigned char *cA = sA + (kt & (STAGES - 1)) * OPA + fA + koff;
      const unsigned char *cB = sB + (kt & (STAGES - 1)) * OPB + fB + koff;
      fa[0] = *reinterpret_cast<const bf16x8_t *>(cA);
#pragma unroll
      for (int t = 0; t < NB; ++t) fb[t] = *reinterpret_cast<const bf16x8_t *>(cB + t * 32 * BK * 2);
#pragma unroll
      for (int t = 1; t < 4; ++t) fa[t] = *reinterpret_cast<const bf16x8_t *>(cA + t * 32 * BK * 2);
    };
    // fragment reads of (kt, half) interleaved with the loads of one operand of a later
    // stage: the three last reads each follow one load, loads left over come after them
    auto lfrag_and_loads = [&](bf16x8_t(&fa)[4], bf16x8_t(&fb)[NB], uint32_t kt, uint32_t koff,
                               const unsigned char *g, lptr_t l, bool operand_a) {
      const unsigned char *cA = sA + (kt & (STAGES - 1)) * OPA + fA + koff;
      const unsigned char *cB = sB + (kt & (STAGES - 1)) * OPB + fB + koff;
      const int nloads = operand_a ? 4 : NB;
      fa[0] = *reinterpret_cast<const bf16x8_t *>(cA);
#pragma unroll
      for (int t = 0; t < NB; ++t) fb[t] = *reinterpret_cast<const bf16x8_t *>(cB + t * 32 * BK * 2);
#pragma unroll
      for (int t = 1; t < 4; ++t) {
        if (t - 1 < nloads) { if (operand_a) load_a(g, l, t - 1); else load_b(g, l, t - 1); }
        fa[t] = *reinterpret_cast<const bf16x8_t *>(cA + t * 32 * BK * 2);
      }
      if (3 < nloads) { if (operand_a) load_a(g, l, 3); else load_b(g, l, 3); }
    };
    auto mma = [&](const bf16x8_t(&fa)[4], const bf16x8_t(&fb)[NB]) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };
    // issue order of one half-step: M = MFMA (mask 0x8), d = LDS read (0x100), G = direct
    // load (0x10).  Four column blocks:  Md Md Md Md Md  MG Md M  MG Md M  MG Md M  MG M
    // two column blocks, A half:  Md Md Md  MGd MGd MGd  MG M;  B half:  Md Md Md  MGd MGd  Md M M
    auto half_step_order = [&](bool operand_a) {
#pragma unroll
      for (int i = 0; i < 1 + NB; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      if constexpr (NB == 4) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      } else if (operand_a) {
#pragma unroll
        for (int i = 0; i < 3; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      }
    };

    // stage 0 has landed once only the two younger stages are in flight
    if (nk > 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS) : "memory");
    else if (nk > 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    lfrag(fa0, fb0, 0, koff0);
    lfrag(fa1, fb1, 0, koff1);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    // Loop invariant at the top of iteration kt: the MFMAs of (kt, first half) are issued,
    // set 1 holds (kt, second half).  An iteration opens with the barrier, so the one wait
    // the compiler places conservatively (at a loop header) coincides with the wait a
    // barrier needs anyway; all other waits sit inside a basic block and name exactly the
    // reads they need.
    uint32_t kt = 0;
    // steady state: stages kt+1 and kt+2 are in flight, stage kt+3 is issued here (its
    // slot in the ring held stage kt-1, whose last reads were issued a whole step ago)
    for (; kt + 3 < nk; ++kt) {
      // one wave polls; the others meet it at the barrier below
      if (ctl.ticks != 0 && wave == 0 && (kt & ctl.mask) == ctl.mask)
        yield_while_preempted(ctl, pause_left);
      // stage kt+1 complete, kt+2 in flight
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
      __syncthreads();  // stage kt+1 is in LDS for everyone; everyone is done with kt-1
      const uint32_t st = (kt + 3) & (STAGES - 1);
      const unsigned char *gA = uA + (uint64_t)(kt + 3) * (BK * 2);
      const unsigned char *gB = uB + (uint64_t)(kt + 3) * (BK * 2);
      lfrag_and_loads(fa0, fb0, kt + 1, koff0, gA, (lptr_t)(sA + st * OPA + ldsA_wave), true);
      mma(fa1, fb1);
      half_step_order(true);
      __builtin_amdgcn_sched_barrier(0);
      lfrag_and_loads(fa1, fb1, kt + 1, koff1, gB, (lptr_t)(sB + st * OPB + ldsB_wave), false);
      mma(fa0, fb0);
      half_step_order(false);
      __builtin_amdgcn_sched_barrier(0);
    }
    // the last steps drain the ring
    for (; kt + 1 < nk; ++kt) {
      if (kt + 2 < nk) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      lfrag(fa0, fb0, kt + 1, koff0);
      __builtin_amdgcn_sched_barrier(0);
      mma(fa1, fb1);
      __builtin_amdgcn_sched_barrier(0);
      lfrag(fa1, fb1, kt + 1, koff1);
      __builtin_amdgcn_sched_barrier(0);
      mma(fa0, fb0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (edge_polls && wave == 0) yield_while_preempted(ctl, pause_left);
    // every wave is past its last fragment read: the ring can be reused as staging space
    __syncthreads();
    mma(fa1, fb1);
    // The accumulators are read below through inline assembly, which the compiler's
    // hazard recogniser cannot see into: keep the last MFMAs from being interleaved with
    // those reads and give the matrix pipe time to retire its last results first.
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // Epilogue.  Lane l, register r of a 32x32 block holds row 8 (r/4) + 4 (l/32) + r%4,
    // column l%32: stored straight from there a wave instruction would write 2 bytes per
    // lane.  Each wave instead stages its 128 x 32 NB sub-tile through LDS, 64 rows at a time
    // (a region of its own, rows 16 bytes more than their length apart so that the two
    // half-waves of a write and the rows of a read fall into different banks), and writes
    // whole row pieces, 16 bytes per lane.  Registers r and r+1 are adjacent rows: one
    // hardware conversion packs both (round to nearest even) and the halves go to LDS
    // separately.  Each accumulator is read where it is used: a wholesale copy of the
    // accumulators into arithmetic registers would double the wave's register footprint,
    // which decides how many other waves fit beside this one.
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    constexpr uint32_t ROWB = 64 * NB;                    // bytes of a sub-tile row
    constexpr uint32_t PITCH = ROWB + 16;
    constexpr uint32_t LPR = ROWB / 16;                   // lanes per row when reading back
    constexpr uint32_t RPI = 64 / LPR;                    // rows per wave instruction
    unsigned char *stage = tally_dyn_lds + wave * (64 * PITCH);
    const uint32_t w_row = (lane >> 5) * 4, w_col = (lane & 31) * 2;
    const uint32_t r_row = lane / LPR, r_chunk = lane % LPR;
    uint16_t *gC = a.C + bz * a.stride_c;
    // an output too large to stay in the 256 MB Infinity Cache beside anything else is
    // written with non-temporal stores in the original form too (2 GB of attention scores:
    // 960 us -> 620 us)
    const bool big_output = (uint64_t)a.m * a.n * a.batch * 2u > (128ull << 20);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int ii = 0; ii < 2; ++ii)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            float v0, v1;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v0) : "a"(acc[2 * h + ii][j][r]));
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v1) : "a"(acc[2 * h + ii][j][r + 1]));
            const f32x2_t p = {v0, v1};
            const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2_t));
            const uint32_t row = ii * 32 + (r >> 2) * 8 + w_row + (r & 3);
            unsigned char *w = stage + row * PITCH + j * 64 + w_col;
            *reinterpret_cast<uint16_t *>(w) = (uint16_t)pk;
            *reinterpret_cast<uint16_t *>(w + PITCH) = (uint16_t)(pk >> 16);
          }
#pragma unroll
      for (uint32_t t = 0; t < 64 / RPI; ++t) {
        const uint32_t row = t * RPI + r_row;
        const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * PITCH + r_chunk * 16);
        const uint32_t grow = by * TILE + wm * 128 + h * 64 + row;
        const uint32_t gcol = bx * TILE_N + wn * 32 * NB + r_chunk * 8;
        if (NT || big_output) {
          const u32x4_nt w = {v.x, v.y, v.z, v.w};
          __builtin_nontemporal_store(w, reinterpret_cast<u32x4_nt *>(gC + (uint64_t)grow * a.n + gcol));
        } else {
          *reinterpret_cast<uint4 *>(gC + (uint64_t)grow * a.n + gcol) = v;
        }
      }
    }
  }
};
using GemmBody = GemmBodyT<4>;
using GemmN128Body = GemmBodyT<2>;

// Same operator with 32x32 output tiles and predicated edges, for small or ragged
// problems (the high-priority inference-like layer), where the grid is far smaller than
// the GPU and every kernel is a chain of memory latencies.  The four waves of a block
// split K between them: wave w multiplies the 16-wide k-chunks w, w+4, w+8, ... (together
// the four waves read whole 128-byte lines of a row), so the serial chain per wave is a
// quarter as long and four times as many waves have loads in flight; the four partial
// tiles are summed through LDS.  Operands come straight from global memory / L2.
struct GemmSmallBody {
  using Args = tally_gemm_bf16_args;
  static constexpr int THREADS = 256;
  // at most 128 registers per lane: that is what a resident 256x256 GEMM tile leaves free
  // on a SIMD, and a high-priority kernel that does not fit beside the paused tiles of a
  // best-effort GEMM waits for them
  static constexpr int MIN_WAVES = 4;
  static constexpr int TILE = 32;
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool YIELDS = false;
  static constexpr bool RANGE = false;
  // the partial sums of consecutive blocks of one workgroup share LDS
  static constexpr bool END_BARRIER = true;
  static constexpr int BATCH = 6;                         // k-chunks requested together per wave

  static __device__ __forceinline__ void run_be(const Args &a, uint32_t x, uint32_t y, uint32_t z) { run(a, x, y, z); }
  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t by, uint32_t bz) {
    __shared__ float s_part[4][16][64];                   // [wave][register][lane]
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    // the wave index decides trip counts below: as a scalar, those become scalar branches
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t K = a.k;
    const uint32_t arow = by * TILE + (lane & 31);
    const uint32_t brow = bx * TILE + (lane & 31);
    const bool aok = arow < a.m, bok = brow < a.n;
    // lane l holds row l%32, elements [8 (l/32), 8 (l/32) + 8) of a 16-wide k-chunk
    const uint32_t LDA = a.lda ? a.lda : K, LDB = a.ldb ? a.ldb : K;
    const uint16_t *pA = a.A + bz * a.stride_a + (uint64_t)(aok ? arow : 0) * LDA + (lane >> 5) * 8;
    const uint16_t *pB = a.Bt + bz * a.stride_b + (uint64_t)(bok ? brow : 0) * LDB + (lane >> 5) * 8;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;

    const uint32_t nchunk = K / 16;                       // this wave takes w, w + 4, ...
    const uint32_t mine = nchunk > wave ? (nchunk - wave + 3) / 4 : 0;
    // chunks [first, first + BATCH) of this wave's share, as far as they exist
    auto request = [&](uint4(&av)[BATCH], uint4(&bv)[BATCH], uint32_t first) {
#pragma unroll
      for (int u = 0; u < BATCH; ++u)
        if (first + u < mine) {
          const uint32_t k0 = (wave + 4 * (first + u)) * 16;
          av[u] = aok ? *reinterpret_cast<const uint4 *>(pA + k0) : zero;
          bv[u] = bok ? *reinterpret_cast<const uint4 *>(pB + k0) : zero;
        }
    };
    auto multiply = [&](const uint4(&av)[BATCH], const uint4(&bv)[BATCH], uint32_t first) {
#pragma unroll
      for (int u = 0; u < BATCH; ++u)
        if (first + u < mine)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av[u]),
                                                        __builtin_bit_cast(bf16x8_t, bv[u]), acc, 0, 0, 0);
    };
    // two register sets: the next batch is on its way while the current one is multiplied
    uint4 a0[BATCH], b0[BATCH], a1[BATCH], b1[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) a0[u] = b0[u] = a1[u] = b1[u] = zero;
    request(a0, b0, 0);
    for (uint32_t c = 0; c < mine; c += 2 * BATCH) {
      request(a1, b1, c + BATCH);
      multiply(a0, b0, c);
      request(a0, b0, c + 2 * BATCH);
      multiply(a1, b1, c + BATCH);
    }

    // sum the four partial tiles: wave w finishes registers 4w .. 4w+3, i.e. rows
    // 8w + 4 (l/32) + {0..3}, column l%32
#pragma unroll
    for (int r = 0; r < 16; ++r) s_part[wave][r][lane] = acc[r];
    __syncthreads();
    uint16_t *gC = a.C + bz * a.stride_c;
    const uint32_t col = bx * TILE + (lane & 31);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t r = wave * 4 + q;
      const float v = (s_part[0][r][lane] + s_part[1][r][lane]) + (s_part[2][r][lane] + s_part[3][r][lane]);
      const uint32_t row = by * TILE + wave * 8 + (lane >> 5) * 4 + q;
      if (row < a.m && col < a.n) gC[(uint64_t)row * a.n + col] = f32_to_bf16(v);
    }
  }
};

// Measured ceiling of the matrix pipe: every wave issues independent 32x32x16 bf16 MFMAs on
// register operands only (no LDS, no memory), one wave per SIMD on every compute unit, as
// a GEMM tile does.  The shader clock is power-managed, so the rate depends on how many
// units are busy and on the operand bits (random bits toggle more than zeros).
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(const uint4 *operands, float *sink,
                                                           uint32_t iters) {
  const uint4 va = operands[threadIdx.x & 63], vb = operands[64 + (threadIdx.x & 63)];
  const bf16x8_t fa = __builtin_bit_cast(bf16x8_t, va), fb = __builtin_bit_cast(bf16x8_t, vb);
  f32x16_t acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace tally
