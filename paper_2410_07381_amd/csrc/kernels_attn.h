// Single-query (decode) attention over a bf16 K/V cache, high-priority path, native form.
//
// The cache is split along the token axis so that heads x splits workgroups keep every
// compute unit streaming HBM: each workgroup scores its token range against the query,
// forms exp(score - local max) weighted sums of V, and writes (max, sum, acc[128]) to
// scratch; a second tiny kernel merges the splits of a head with the usual max/sum
// rescaling.  16 lanes cover one token's 128-wide row with 16-byte loads, so a wave load
// touches four whole 256-byte rows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../include/tally.h"
#include "kernels_stream.h"

namespace tally {

constexpr uint32_t kAttnSplits = 16;
constexpr uint32_t kAttnDim = 128;
constexpr uint32_t kAttnMaxChunk = 2048;                  // tokens per workgroup
constexpr uint32_t kAttnRec = kAttnDim + 2;               // floats per partial record

inline size_t attn_decode_scratch_bytes(uint32_t heads) {
  return (size_t)heads * kAttnSplits * kAttnRec * sizeof(float);
}

__device__ __forceinline__ void unpack8(uint4 u, float (&f)[8]) {
  f[0] = bf16_lo(u.x); f[1] = bf16_hi(u.x); f[2] = bf16_lo(u.y); f[3] = bf16_hi(u.y);
  f[4] = bf16_lo(u.z); f[5] = bf16_hi(u.z); f[6] = bf16_lo(u.w); f[7] = bf16_hi(u.w);
}

__global__ __launch_bounds__(256, 4) void attn_decode_partial(tally_attn_decode_args a, uint32_t chunk,
                                                           uint32_t urgent) {
  if (urgent) __builtin_amdgcn_s_setprio(3);
  __shared__ float s_score[kAttnMaxChunk];
  __shared__ float s_red[4];
  __shared__ float s_acc[4][kAttnDim];
  const uint32_t split = blockIdx.x, h = blockIdx.y;
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t grp = lane >> 4, sub = lane & 15;
  const uint32_t t0 = split * chunk;
  const uint32_t t1 = min(t0 + chunk, a.tokens);
  const uint32_t cnt = t1 > t0 ? t1 - t0 : 0;
  const uint64_t row = (uint64_t)a.heads * kAttnDim;       // elements between tokens
  const uint16_t *Kh = a.K + (uint64_t)h * kAttnDim + sub * 8;
  const uint16_t *Vh = a.V + (uint64_t)h * kAttnDim + sub * 8;
  const uint4 qq = *reinterpret_cast<const uint4 *>(a.q + (uint64_t)h * kAttnDim + sub * 8);
  const float scale = 0.08838834764831845f;                // 1 / sqrt(128)

  // Both passes take their tokens eight at a time per 16-lane group and issue the eight
  // 16-byte loads before they use the first: with one load in flight per pass of the loop a
  // workgroup was a chain of sixteen memory latencies for its 128 tokens (the whole kernel
  // 11 us for 33.6 MB, twice that from a cold cache), and beside the paused tiles of a
  // best-effort GEMM there are few other waves on the compute unit to hide them.
  constexpr int U = 8;
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  // pass 1: scores of this workgroup's tokens
  float mloc = -INFINITY;
  for (uint32_t tb = wave * 4 + grp; tb < chunk; tb += 16 * U) {  // uniform trip count per wave
    uint4 kk[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t t = tb + 16 * u;
      kk[u] = zero4;
      if (t < cnt) kk[u] = *reinterpret_cast<const uint4 *>(Kh + (uint64_t)(t0 + t) * row);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t t = tb + 16 * u;
      if (t < chunk) {                                     // chunk is a multiple of 16: wave-uniform
        float s = GemvBody::dot8(kk[u], qq, 0.f);
        s += __shfl_xor(s, 8, kWave);
        s += __shfl_xor(s, 4, kWave);
        s += __shfl_xor(s, 2, kWave);
        s += __shfl_xor(s, 1, kWave);
        s = (t < cnt) ? s * scale : -INFINITY;
        if (sub == 0) s_score[t] = s;
        mloc = fmaxf(mloc, s);
      }
    }
  }
  mloc = wave_max(mloc);
  if (lane == 0) s_red[wave] = mloc;
  __syncthreads();
  const float m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));

  // pass 2: weights and weighted sum of V
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (uint32_t tb = wave * 4 + grp; tb < chunk; tb += 16 * U) {
    uint4 vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t t = tb + 16 * u;
      vv[u] = zero4;
      if (t < cnt) vv[u] = *reinterpret_cast<const uint4 *>(Vh + (uint64_t)(t0 + t) * row);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t t = tb + 16 * u;
      // a token beyond the range has weight 0 and a zero row: it adds nothing
      const float p = (t < cnt) ? __expf(s_score[t < cnt ? t : 0u] - m) : 0.f;
      const uint4 r = vv[u];
      acc[0] = __builtin_fmaf(p, bf16_lo(r.x), acc[0]);
      acc[1] = __builtin_fmaf(p, bf16_hi(r.x), acc[1]);
      acc[2] = __builtin_fmaf(p, bf16_lo(r.y), acc[2]);
      acc[3] = __builtin_fmaf(p, bf16_hi(r.y), acc[3]);
      acc[4] = __builtin_fmaf(p, bf16_lo(r.z), acc[4]);
      acc[5] = __builtin_fmaf(p, bf16_hi(r.z), acc[5]);
      acc[6] = __builtin_fmaf(p, bf16_lo(r.w), acc[6]);
      acc[7] = __builtin_fmaf(p, bf16_hi(r.w), acc[7]);
      l += p;
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    acc[e] += __shfl_xor(acc[e], 16, kWave);
    acc[e] += __shfl_xor(acc[e], 32, kWave);
  }
  l += __shfl_xor(l, 16, kWave);
  l += __shfl_xor(l, 32, kWave);
  __syncthreads();                                         // s_red reuse
  if (grp == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[wave][sub * 8 + e] = acc[e];
  }
  if (lane == 0) s_red[wave] = l;
  __syncthreads();
  float *rec = reinterpret_cast<float *>(a.scratch) + ((uint64_t)h * kAttnSplits + split) * kAttnRec;
  if (tid < kAttnDim)
    rec[2 + tid] = (s_acc[0][tid] + s_acc[1][tid]) + (s_acc[2][tid] + s_acc[3][tid]);
  if (tid == 0) {
    rec[0] = m;
    rec[1] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
  }
}

__global__ __launch_bounds__(128) void attn_decode_combine(tally_attn_decode_args a) {
  const uint32_t h = blockIdx.x, d = threadIdx.x;
  const float *rec = reinterpret_cast<const float *>(a.scratch) + (uint64_t)h * kAttnSplits * kAttnRec;
  float M = -INFINITY;
#pragma unroll
  for (uint32_t s = 0; s < kAttnSplits; ++s) M = fmaxf(M, rec[s * kAttnRec]);
  float num = 0.f, den = 0.f;
#pragma unroll
  for (uint32_t s = 0; s < kAttnSplits; ++s) {
    float ms = rec[s * kAttnRec];
    float w = (ms == -INFINITY) ? 0.f : __expf(ms - M);
    num = __builtin_fmaf(w, rec[s * kAttnRec + 2 + d], num);
    den = __builtin_fmaf(w, rec[s * kAttnRec + 1], den);
  }
  a.out[(uint64_t)h * kAttnDim + d] = f32_to_bf16(num / den);
}

inline hipError_t attn_decode_init() { return hipSuccess; }

inline hipError_t launch_attn_decode(hipStream_t s, const void *args, tally_dim3, uint32_t urgent) {
  tally_attn_decode_args a;
  memcpy(&a, args, sizeof(a));
  uint32_t chunk = (a.tokens + kAttnSplits - 1) / kAttnSplits;
  chunk = (chunk + 15u) & ~15u;
  if (chunk > kAttnMaxChunk) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_decode_partial, dim3(kAttnSplits, a.heads), dim3(256), 0, s, a, chunk,
                     urgent);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_decode_combine, dim3(a.heads), dim3(128), 0, s, a);
  return hipGetLastError();
}

}  // namespace tally
