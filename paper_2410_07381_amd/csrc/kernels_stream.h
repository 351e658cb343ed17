// HBM-streaming workload kernels as logical-block bodies: SAXPY, sum reduction, GEMV,
// row softmax, row LayerNorm.  All are bandwidth-bound: 16-byte coalesced loads, one
// 64-lane wave per row for the row-wise kernels, cross-lane reductions without LDS
// where a wave owns the whole row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tally.h"

namespace tally {

constexpr int kThreads = 256;
constexpr int kWave = 64;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
// Best-effort forms stream their data with non-temporal accesses (NT): what a best-effort
// kernel reads once and writes once would otherwise push the high-priority job's weights
// and caches out of the L2s and the 256 MB Infinity Cache between two of its requests
// (measured: a decode step beside a streaming softmax took 65 us instead of 41 on the
// device with ordinary accesses, 36 us with non-temporal ones).  The original form of a
// kernel keeps ordinary accesses.
typedef float f32x4_nt __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ float4 ld4(const float *p) {
  if constexpr (NT) {
    const f32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_nt *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
  } else {
    return *reinterpret_cast<const float4 *>(p);
  }
}
template <bool NT>
__device__ __forceinline__ void st4(float *p, float4 v) {
  if constexpr (NT) {
    const f32x4_nt w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<f32x4_nt *>(p));
  } else {
    *reinterpret_cast<float4 *>(p) = v;
  }
}
template <bool NT>
__device__ __forceinline__ float ld1(const float *p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT>
__device__ __forceinline__ void st1(float *p, float v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;  // NaN
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// ---- SAXPY: thread t of block b handles element 256 b + t ----------------------------
struct SaxpyBody {
  using Args = tally_saxpy_args;
  static constexpr int THREADS = kThreads;
  static constexpr int MIN_WAVES = 4;
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool YIELDS = false;
  static constexpr bool END_BARRIER = false;
  static constexpr bool RANGE = true;
  template <bool NT>
  static __device__ __forceinline__ void run_t(const Args &a, uint32_t bx) {
    uint32_t i = bx * kThreads + threadIdx.x;
    if (i < a.n) st1<NT>(a.y + i, __builtin_fmaf(a.a, ld1<NT>(a.x + i), ld1<NT>(a.y + i)));
  }
  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<false>(a, bx); }
  static __device__ __forceinline__ void run_be(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<true>(a, bx); }
  // Logical blocks [first, last) of the (one-dimensional) grid in one go, for a worker that
  // fetched several consecutive task indices: the same elements get the same arithmetic as
  // block by block, but the loads of eight blocks are in flight together instead of one
  // block's loads waiting for the previous block's store.
  static __device__ __forceinline__ void run_range(const Args &a, uint32_t first, uint32_t last) {
    const float *__restrict__ x = a.x;
    float *__restrict__ y = a.y;
    const uint32_t end = last * kThreads < a.n ? last * kThreads : a.n;
    uint32_t i = first * kThreads + threadIdx.x;
    for (; i + 7 * kThreads < end; i += 8 * kThreads) {
      float xv[8], yv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) { xv[u] = ld1<true>(x + i + u * kThreads); yv[u] = ld1<true>(y + i + u * kThreads); }
#pragma unroll
      for (int u = 0; u < 8; ++u) st1<true>(y + i + u * kThreads, __builtin_fmaf(a.a, xv[u], yv[u]));
    }
    for (; i < end; i += kThreads) st1<true>(y + i, __builtin_fmaf(a.a, ld1<true>(x + i), ld1<true>(y + i)));
  }
};

// ---- sum reduction: block b -> partial[b] over 4096 consecutive elements --------------
struct ReduceSumBody {
  using Args = tally_reduce_sum_args;
  static constexpr int THREADS = kThreads;
  static constexpr int MIN_WAVES = 4;
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool YIELDS = false;
  static constexpr bool RANGE = true;
  static constexpr bool END_BARRIER = false;
  static constexpr uint32_t PER_BLOCK = 4096;
  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<false>(a, bx); }
  static __device__ __forceinline__ void run_be(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<true>(a, bx); }
  template <bool NT>
  static __device__ __forceinline__ void run_t(const Args &a, uint32_t bx) {
    // two sets of wave partials, alternating with the block index: a worker that runs
    // consecutive blocks back to back then needs no barrier between them (the barrier
    // below already keeps any wave at most one block ahead of the reader)
    __shared__ float s_part2[2][kThreads / kWave];
    float *s_part = s_part2[bx & 1];
    const uint64_t base = (uint64_t)bx * PER_BLOCK;
    float s = 0.f;
    if (base + PER_BLOCK <= a.n) {
      const float *p = a.x + base + 4 * threadIdx.x;
      float4 v0 = ld4<NT>(p), v1 = ld4<NT>(p + 1024), v2 = ld4<NT>(p + 2048), v3 = ld4<NT>(p + 3072);
      s = ((v0.x + v0.y) + (v0.z + v0.w)) + ((v1.x + v1.y) + (v1.z + v1.w)) +
          (((v2.x + v2.y) + (v2.z + v2.w)) + ((v3.x + v3.y) + (v3.z + v3.w)));
    } else {
      for (uint64_t i = base + threadIdx.x; i < a.n; i += kThreads) s += a.x[i];
    }
    s = wave_sum(s);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = s;
    __syncthreads();
    if (threadIdx.x == 0) a.partial[bx] = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
  }
  // Consecutive blocks [first, last) for a worker that fetched several task indices: four
  // blocks at a time, their 64 KB requested together before any of them is reduced, and one
  // barrier for the four (a persistent worker has far fewer blocks in flight per compute unit
  // than the hardware keeps when it dispatches the original grid, so it has to ask for more
  // per block-time to keep the memory system as busy).  Per block the same sums in the same
  // order as run().
  static __device__ __forceinline__ void run_range(const Args &a, uint32_t first, uint32_t last) {
    __shared__ float s_quad[2][4][kThreads / kWave];
    const uint32_t t = threadIdx.x;
    uint32_t b = first;
    for (uint32_t it = 0; b + 4 <= last && ((uint64_t)b + 4) * PER_BLOCK <= a.n; b += 4, ++it) {
      float4 v[4][4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float *p = a.x + (uint64_t)(b + q) * PER_BLOCK + 4 * t;
        v[q][0] = ld4<true>(p); v[q][1] = ld4<true>(p + 1024); v[q][2] = ld4<true>(p + 2048); v[q][3] = ld4<true>(p + 3072);
      }
      float (*part)[kThreads / kWave] = s_quad[it & 1];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float s = ((v[q][0].x + v[q][0].y) + (v[q][0].z + v[q][0].w)) +
                  ((v[q][1].x + v[q][1].y) + (v[q][1].z + v[q][1].w)) +
                  (((v[q][2].x + v[q][2].y) + (v[q][2].z + v[q][2].w)) +
                   ((v[q][3].x + v[q][3].y) + (v[q][3].z + v[q][3].w)));
        s = wave_sum(s);
        if ((t & (kWave - 1)) == 0) part[q][t / kWave] = s;
      }
      __syncthreads();   // (the other buffer is free again: its reader is past this barrier)
      if (t < 4) a.partial[b + t] = (part[t][0] + part[t][1]) + (part[t][2] + part[t][3]);
    }
    for (; b < last; ++b) run_t<true>(a, b);
  }
};

struct ReduceFinalBody {
  using Args = tally_reduce_final_args;
  static constexpr int THREADS = kThreads;
  static constexpr int MIN_WAVES = 4;
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool YIELDS = false;
  static constexpr bool RANGE = false;
  static constexpr bool END_BARRIER = true;   // s_d is reused by the next block
  static __device__ __forceinline__ void run_be(const Args &a, uint32_t x, uint32_t y, uint32_t z) { run(a, x, y, z); }
  static __device__ __forceinline__ void run(const Args &a, uint32_t, uint32_t, uint32_t) {
    __shared__ double s_d[kThreads];
    double s = 0.0;
    for (uint32_t i = threadIdx.x; i < a.count; i += kThreads) s += (double)a.partial[i];
    s_d[threadIdx.x] = s;
    __syncthreads();
    for (int o = kThreads / 2; o > 0; o >>= 1) {
      if ((int)threadIdx.x < o) s_d[threadIdx.x] += s_d[threadIdx.x + o];
      __syncthreads();
    }
    if (threadIdx.x == 0) *a.total = s_d[0];
  }
};

// ---- GEMV: one wave per output row, 16-byte loads along K -----------------------------
struct GemvBody {
  using Args = tally_gemv_bf16_args;
  static constexpr int THREADS = kThreads;
  static constexpr int MIN_WAVES = 8;   // <= 64 registers: two waves fit beside a GEMM tile
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool YIELDS = false;
  static constexpr bool RANGE = false;
  static constexpr bool END_BARRIER = false;
  // 8 bf16 products per 16-byte pair with four packed dot-product instructions (fp32
  // accumulate): a sixth of the vector-ALU work of unpack + fma, which matters because
  // a high-priority GEMV may share its SIMDs with a best-effort GEMM's MFMA stream
  static __device__ __forceinline__ float dot8(uint4 w, uint4 x, float s) {
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x),
                                        __builtin_bit_cast(bf16x2_t, x.x), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y),
                                        __builtin_bit_cast(bf16x2_t, x.y), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z),
                                        __builtin_bit_cast(bf16x2_t, x.z), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w),
                                        __builtin_bit_cast(bf16x2_t, x.w), s, false);
    return s;
  }
  // (the best-effort forms keep four loads in flight: their loop has no registers to spare)
  static __device__ __forceinline__ void run_be(const Args &a, uint32_t x, uint32_t y, uint32_t z) { run_t<false>(a, x, y, z); }
  static __device__ __forceinline__ void run(const Args &a, uint32_t x, uint32_t y, uint32_t z) { run_t<true>(a, x, y, z); }
  template <bool DEEP>
  static __device__ __forceinline__ void run_t(const Args &a, uint32_t bx, uint32_t, uint32_t) {
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t row = bx * 4 + threadIdx.x / kWave;
    if (row >= a.n) return;  // wave-uniform; the body holds no barrier
    const uint32_t nvec = a.k / 8;
    const uint4 *w = reinterpret_cast<const uint4 *>(a.W + (uint64_t)row * a.k);
    const uint4 *x = reinterpret_cast<const uint4 *>(a.x);
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
    uint32_t v = lane;
    // Eight 16-byte loads of the row in flight per lane (8 KB per wave; a 4096-wide row is
    // one such batch).  Beside the paused tiles of a best-effort GEMM only two of these
    // waves fit on a SIMD, and with four loads each the eight waves of a compute unit had
    // 32 KB on their way where the HBM's latency times the unit's share of its bandwidth
    // asks for ~45 KB: the decode-like request ran at 4.3 TB/s co-located against 5.6 alone.
    // The operand x comes from the caches; its loads are taken four at a time to stay
    // within the 64 registers that let two waves fit.
    for (; DEEP && v + 7 * kWave < nvec; v += 8 * kWave) {
      const uint4 w0 = w[v], w1 = w[v + kWave], w2 = w[v + 2 * kWave], w3 = w[v + 3 * kWave];
      const uint4 w4 = w[v + 4 * kWave], w5 = w[v + 5 * kWave], w6 = w[v + 6 * kWave], w7 = w[v + 7 * kWave];
      uint4 x0 = x[v], x1 = x[v + kWave], x2 = x[v + 2 * kWave], x3 = x[v + 3 * kWave];
      acc0 = dot8(w0, x0, acc0);
      acc1 = dot8(w1, x1, acc1);
      acc2 = dot8(w2, x2, acc2);
      acc3 = dot8(w3, x3, acc3);
      x0 = x[v + 4 * kWave]; x1 = x[v + 5 * kWave]; x2 = x[v + 6 * kWave]; x3 = x[v + 7 * kWave];
      acc0 = dot8(w4, x0, acc0);
      acc1 = dot8(w5, x1, acc1);
      acc2 = dot8(w6, x2, acc2);
      acc3 = dot8(w7, x3, acc3);
    }
    for (; v + 3 * kWave < nvec; v += 4 * kWave) {
      uint4 w0 = w[v], w1 = w[v + kWave], w2 = w[v + 2 * kWave], w3 = w[v + 3 * kWave];
      acc0 = dot8(w0, x[v], acc0);
      acc1 = dot8(w1, x[v + kWave], acc1);
      acc2 = dot8(w2, x[v + 2 * kWave], acc2);
      acc3 = dot8(w3, x[v + 3 * kWave], acc3);
    }
    for (; v < nvec; v += kWave) acc0 = dot8(w[v], x[v], acc0);
    float s = wave_sum((acc0 + acc1) + (acc2 + acc3));
    if (lane == 0) a.y[row] = f32_to_bf16(s);
  }
};

// ---- row-wise kernels: a wave keeps its row in registers as NV float4 per lane --------
template <int NV, bool NT>
__device__ __forceinline__ void load_row(const float *row, uint32_t cols, uint32_t lane,
                                         float4 (&v)[NV], float fill) {
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    uint32_t c = (i * kWave + lane) * 4;
    v[i] = (c < cols) ? ld4<NT>(row + c) : make_float4(fill, fill, fill, fill);
  }
}

template <int NV, bool NT>
__device__ __forceinline__ void softmax_row(const float *x, float *y, uint32_t cols, uint32_t lane) {
  float4 v[NV];
  load_row<NV, NT>(x, cols, lane, v, -INFINITY);
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) m = fmaxf(m, fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w)));
  m = wave_max(m);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    v[i].x = __expf(v[i].x - m); v[i].y = __expf(v[i].y - m);
    v[i].z = __expf(v[i].z - m); v[i].w = __expf(v[i].w - m);
    s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  }
  s = wave_sum(s);
  const float inv = 1.0f / s;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    uint32_t c = (i * kWave + lane) * 4;
    if (c < cols) st4<NT>(y + c, make_float4(v[i].x * inv, v[i].y * inv, v[i].z * inv, v[i].w * inv));
  }
}

// Rows wider than 4096 would need more than 64 registers per lane to stay resident, and
// the widest instantiation sets the register allocation (hence the occupancy) of the
// whole kernel; such rows are walked three times instead and come from cache after the
// first pass.
__device__ __forceinline__ void softmax_row_streamed(const float *x, float *y, uint32_t cols,
                                                     uint32_t lane) {
  float m = -INFINITY;
  for (uint32_t c = lane * 4; c < cols; c += kWave * 4) {
    float4 v = *reinterpret_cast<const float4 *>(x + c);
    m = fmaxf(m, fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
  }
  m = wave_max(m);
  float s = 0.f;
  for (uint32_t c = lane * 4; c < cols; c += kWave * 4) {
    float4 v = *reinterpret_cast<const float4 *>(x + c);
    s += (__expf(v.x - m) + __expf(v.y - m)) + (__expf(v.z - m) + __expf(v.w - m));
  }
  const float inv = 1.0f / wave_sum(s);
  for (uint32_t c = lane * 4; c < cols; c += kWave * 4) {
    float4 v = *reinterpret_cast<const float4 *>(x + c);
    *reinterpret_cast<float4 *>(y + c) = make_float4(__expf(v.x - m) * inv, __expf(v.y - m) * inv,
                                                     __expf(v.z - m) * inv, __expf(v.w - m) * inv);
  }
}

// MAXNV bounds the widest row instantiated (in float4 per lane): the widest instantiation
// sets the register allocation of the whole kernel, so rows of up to 1024 columns get a
// kernel of their own that needs a quarter of the registers.  A high-priority kernel over
// narrow rows then fits several waves per SIMD beside paused best-effort workgroups.
template <int MAXNV>
struct SoftmaxBodyT {
  using Args = tally_softmax_f32_args;
  static constexpr int THREADS = kThreads;
  static constexpr int MIN_WAVES = MAXNV <= 4 ? 8 : 4;
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool YIELDS = false;
  static constexpr bool RANGE = false;
  static constexpr bool END_BARRIER = false;
  static constexpr uint32_t MAX_COLS = MAXNV * kWave * 4;   // widest row held in registers
  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<false>(a, bx); }
  static __device__ __forceinline__ void run_be(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<true>(a, bx); }
  template <bool NT>
  static __device__ __forceinline__ void run_t(const Args &a, uint32_t bx) {
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t row = bx * 4 + threadIdx.x / kWave;
    if (row >= a.rows) return;
    const float *x = a.x + (uint64_t)row * a.cols;
    float *y = a.y + (uint64_t)row * a.cols;
    if (a.cols <= 256) softmax_row<1, NT>(x, y, a.cols, lane);
    else if (a.cols <= 512) softmax_row<2, NT>(x, y, a.cols, lane);
    else if (a.cols <= 1024) softmax_row<4, NT>(x, y, a.cols, lane);
    else if constexpr (MAXNV >= 16) {
      if (a.cols <= 2048) softmax_row<8, NT>(x, y, a.cols, lane);
      else if (a.cols <= 4096) softmax_row<16, NT>(x, y, a.cols, lane);
      else softmax_row_streamed(x, y, a.cols, lane);   // (re-read twice: ordinary accesses)
    }
  }
};
using SoftmaxBody = SoftmaxBodyT<16>;
using SoftmaxNarrowBody = SoftmaxBodyT<4>;

template <int NV, bool NT>
__device__ __forceinline__ void layernorm_row(const float *x, const float *g, const float *b,
                                              float *y, uint32_t cols, float eps, uint32_t lane) {
  float4 v[NV];
  load_row<NV, NT>(x, cols, lane, v, 0.f);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  const float mu = wave_sum(s) / (float)cols;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    uint32_t c = (i * kWave + lane) * 4;
    if (c < cols) {
      float dx = v[i].x - mu, dy = v[i].y - mu, dz = v[i].z - mu, dw = v[i].w - mu;
      q += (dx * dx + dy * dy) + (dz * dz + dw * dw);
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)cols + eps);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    uint32_t c = (i * kWave + lane) * 4;
    if (c < cols) {
      float4 gg = *reinterpret_cast<const float4 *>(g + c);
      float4 bb = *reinterpret_cast<const float4 *>(b + c);
      st4<NT>(y + c, make_float4(
          __builtin_fmaf((v[i].x - mu) * rstd, gg.x, bb.x),
          __builtin_fmaf((v[i].y - mu) * rstd, gg.y, bb.y),
          __builtin_fmaf((v[i].z - mu) * rstd, gg.z, bb.z),
          __builtin_fmaf((v[i].w - mu) * rstd, gg.w, bb.w)));
    }
  }
}

__device__ __forceinline__ void layernorm_row_streamed(const float *x, const float *g,
                                                       const float *b, float *y, uint32_t cols,
                                                       float eps, uint32_t lane) {
  float s = 0.f;
  for (uint32_t c = lane * 4; c < cols; c += kWave * 4) {
    float4 v = *reinterpret_cast<const float4 *>(x + c);
    s += (v.x + v.y) + (v.z + v.w);
  }
  const float mu = wave_sum(s) / (float)cols;
  float q = 0.f;
  for (uint32_t c = lane * 4; c < cols; c += kWave * 4) {
    float4 v = *reinterpret_cast<const float4 *>(x + c);
    float dx = v.x - mu, dy = v.y - mu, dz = v.z - mu, dw = v.w - mu;
    q += (dx * dx + dy * dy) + (dz * dz + dw * dw);
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)cols + eps);
  for (uint32_t c = lane * 4; c < cols; c += kWave * 4) {
    float4 v = *reinterpret_cast<const float4 *>(x + c);
    float4 gg = *reinterpret_cast<const float4 *>(g + c);
    float4 bb = *reinterpret_cast<const float4 *>(b + c);
    *reinterpret_cast<float4 *>(y + c) =
        make_float4(__builtin_fmaf((v.x - mu) * rstd, gg.x, bb.x),
                    __builtin_fmaf((v.y - mu) * rstd, gg.y, bb.y),
                    __builtin_fmaf((v.z - mu) * rstd, gg.z, bb.z),
                    __builtin_fmaf((v.w - mu) * rstd, gg.w, bb.w));
  }
}

template <int MAXNV>
struct LayerNormBodyT {
  using Args = tally_layernorm_f32_args;
  static constexpr int THREADS = kThreads;
  static constexpr int MIN_WAVES = MAXNV <= 4 ? 8 : 2;
  static constexpr unsigned DYN_LDS = 0;
  static constexpr bool YIELDS = false;
  static constexpr bool RANGE = false;
  static constexpr bool END_BARRIER = false;
  static constexpr uint32_t MAX_COLS = MAXNV * kWave * 4;
  static __device__ __forceinline__ void run(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<false>(a, bx); }
  static __device__ __forceinline__ void run_be(const Args &a, uint32_t bx, uint32_t, uint32_t) { run_t<true>(a, bx); }
  template <bool NT>
  static __device__ __forceinline__ void run_t(const Args &a, uint32_t bx) {
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t row = bx * 4 + threadIdx.x / kWave;
    if (row >= a.rows) return;
    const float *x = a.x + (uint64_t)row * a.cols;
    float *y = a.y + (uint64_t)row * a.cols;
    if (a.cols <= 256) layernorm_row<1, NT>(x, a.gamma, a.beta, y, a.cols, a.eps, lane);
    else if (a.cols <= 512) layernorm_row<2, NT>(x, a.gamma, a.beta, y, a.cols, a.eps, lane);
    else if (a.cols <= 1024) layernorm_row<4, NT>(x, a.gamma, a.beta, y, a.cols, a.eps, lane);
    else if constexpr (MAXNV >= 16) {
      if (a.cols <= 2048) layernorm_row<8, NT>(x, a.gamma, a.beta, y, a.cols, a.eps, lane);
      else if (a.cols <= 4096) layernorm_row<16, NT>(x, a.gamma, a.beta, y, a.cols, a.eps, lane);
      else layernorm_row_streamed(x, a.gamma, a.beta, y, a.cols, a.eps, lane);
    }
  }
};
using LayerNormBody = LayerNormBodyT<16>;
using LayerNormNarrowBody = LayerNormBodyT<4>;

}  // namespace tally
