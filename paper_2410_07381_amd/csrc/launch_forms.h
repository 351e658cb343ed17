// The three launch forms of a best-effort kernel, generated from one logical-block body.
//
// A Body is a struct with
//   using Args = <POD passed by value to the kernel>;
//   static constexpr int THREADS;            threads per logical block
//   static constexpr int MIN_WAVES;          waves per SIMD the compiler must leave room for
//   static constexpr unsigned DYN_LDS;       dynamic LDS bytes the body needs
//   static constexpr bool END_BARRIER;       true if consecutive blocks run by one workgroup
//                                            would race on workgroup-shared state
//   static constexpr bool YIELDS;            true if the body offers run_yielding(), which
//                                            pauses inside the block while preempted
//   static __device__ void run(const Args&, uint32_t bx, uint32_t by, uint32_t bz);
// run() performs the work of original block (bx,by,bz); every thread of the workgroup
// calls it and returns from it (no early exit), so the workgroup-wide barriers of the
// persistent-worker loop are reached by all threads (Section 4.1: divergent barriers
// stall a kernel for ever; hand-written bodies handle ragged tails by predication).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tally.h"

namespace tally {

constexpr uint32_t kStop = 0xFFFFFFFFu;

// Device-side control block of one persistent-worker launch segment.
struct PtbCtl {
  uint32_t *counter;        // device: global task counter (next task index)
  uint32_t *dev_flag;       // device, 8-byte aligned: [0] epoch of the last preemption relayed,
                            // [1] epoch of the last segment whose grid was exhausted
  uint32_t *exited;         // device: workers that have exited, summed over all segments
  const uint32_t *host_flag;  // pinned host memory: epoch the host wants preempted
  unsigned long long *host_status;  // pinned: (epoch << 32 | progress) once drained
  uint32_t *host_live;      // pinned: progress mirrored while running
  uint32_t *host_raw;       // pinned: raw counter value at the drain (written before status)
  tally_cover_rec *cover;   // device, may be null
  uint32_t total;           // logical blocks in the grid
  uint32_t limit;           // workers treat this as the end of the grid (== total normally)
  uint32_t epoch;           // id of this launch segment, unique for the life of the slot
  uint32_t exit_target;     // value of *exited after the last worker of this segment leaves
  uint32_t counter_base;    // raw counter value that stands for task index 0 of this job
  uint32_t workers;
  uint32_t chunk;           // task indices per fetch
  uint32_t segment;         // 0-based segment number, for the coverage records
  uint32_t gx, gy;          // logical grid extents (x fastest)
  uint32_t yield_ticks;     // longest pause inside a block, in 10 ns wall-clock ticks (0: never)
  uint32_t *flag_copies;    // device: kFlagCopies copies of dev_flag[0], 128 B apart, for the
                            // mid-block polls (one address serves only ~80 M coherent scalar
                            // loads per second, whoever asks)
};
constexpr uint32_t kFlagCopies = 64;
constexpr uint32_t kFlagCopyStride = 32;  // in 32-bit words

struct SliceCtl {
  tally_cover_rec *cover;
  uint32_t offset;          // first logical block of this sub-kernel
  uint32_t gx, gy;
  uint32_t segment;
};

__device__ __forceinline__ void delinearize(uint32_t idx, uint32_t gx, uint32_t gy, uint32_t &bx,
                                            uint32_t &by, uint32_t &bz) {
  bx = idx % gx;
  uint32_t r = idx / gx;
  by = r % gy;
  bz = r / gy;
}

__device__ __forceinline__ void record(tally_cover_rec *cover, uint32_t idx, uint32_t bx,
                                       uint32_t by, uint32_t bz, uint32_t segment,
                                       uint32_t worker) {
  if (cover != nullptr && threadIdx.x == 0) {
    tally_cover_rec *r = cover + idx;
    atomicAdd(&r->count, 1u);
    r->bx = bx; r->by = by; r->bz = bz; r->segment = segment; r->worker = worker;
  }
}

// ---- original form -------------------------------------------------------------------
// `urgent` marks a launch on the high-priority stream: its waves raise their own issue
// priority so that, where they share a SIMD with a best-effort wave that is still
// finishing its block, the arbiter picks their instructions first.
template <class Body>
__global__ __launch_bounds__(Body::THREADS, Body::MIN_WAVES) void native_kernel(typename Body::Args args,
                                                               uint32_t urgent) {
  if (urgent) __builtin_amdgcn_s_setprio(3);
  Body::run(args, blockIdx.x, blockIdx.y, blockIdx.z);
}



// ---- sliced form: logical block = offset + blockIdx (Section 4.1, slicing) -----------
template <class Body>
__device__ __forceinline__ void sliced_body(const typename Body::Args &args, const SliceCtl &ctl) {
  uint32_t idx = ctl.offset + blockIdx.x, bx, by, bz;
  delinearize(idx, ctl.gx, ctl.gy, bx, by, bz);
  Body::run(args, bx, by, bz);
  record(ctl.cover, idx, bx, by, bz, ctl.segment, blockIdx.x);
}
template <class Body>
__global__ __launch_bounds__(Body::THREADS, Body::MIN_WAVES) void sliced_kernel(typename Body::Args args,
                                                               SliceCtl ctl) {
  sliced_body<Body>(args, ctl);
}

// ---- persistent-worker form (Section 4.1, preemption) --------------------------------
// The host raises the flag with one store to pinned host memory (cheap to write, but a
// load from it crosses PCIe, far too slow for hundreds of workers to poll every
// iteration).  A one-wave relay kernel, launched just before the workers on a stream of
// its own, polls that word, copies every change of it into a device-memory flag the
// workers can poll cheaply, and mirrors the progress back to the host.  It leaves when
// every worker of the segment has exited, so its lifetime is bounded by the workers',
// which depend on nothing.
//
// The relay polls with scalar loads that bypass the scalar cache: a vector load that
// waits a microsecond on PCIe sits in the compute unit's vector-memory return queue in
// front of the loads of whatever worker shares that unit (measured: that worker's GEMM
// tile ran 20 % longer, and with it the whole kernel); the scalar path is separate.
__device__ __forceinline__ uint32_t scalar_load_coherent(const uint32_t *p) {
  uint32_t v;
  asm volatile("s_load_dword %0, %1, 0x0 glc\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
  return v;
}

constexpr unsigned long long kRelayGiveUpTicks = 2000000ull;  // 20 ms of the 100 MHz clock

__global__ __launch_bounds__(64) void relay_kernel(PtbCtl c) {
  uint32_t last = 0xFFFFFFFFu;
  // The relay is launched before its workers.  Where the two cannot run side by side
  // (kernels executed strictly one after another) the workers cannot start until the
  // relay has ended: it leaves when neither the task counter nor the exit counter has
  // moved for 20 ms, and that launch segment then runs without the means to preempt it.
  const unsigned long long born = wall_clock64();
  const uint32_t ctr0 = scalar_load_coherent(c.counter), gone0 = scalar_load_coherent(c.exited);
  bool alive = false;
  for (uint32_t n = 0;; ++n) {
    // forward every change of the host's word: a request (the segment's epoch) and, later,
    // its withdrawal, which lets workers that paused inside a long block carry on
    uint32_t want = scalar_load_coherent(c.host_flag);
    if (want != last) {
      if (threadIdx.x == 0)
        __hip_atomic_store(c.dev_flag, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (c.flag_copies != nullptr && threadIdx.x < kFlagCopies)
        __hip_atomic_store(c.flag_copies + threadIdx.x * kFlagCopyStride, want, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      last = want;
    }
    // the counters of a slot only ever grow (they are never reset), so a relay that
    // starts late, even after its workers are long gone, still sees the target passed
    uint32_t gone = scalar_load_coherent(c.exited);
    if ((n & 255u) == 255u)  // and, now and then, through the path the workers' atomics use
      gone = __hip_atomic_load(c.exited, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((int32_t)(gone - c.exit_target) >= 0) return;
    if ((n & 15u) == 0u) {
      const uint32_t raw = scalar_load_coherent(c.counter);
      if (raw != ctr0 || gone != gone0) alive = true;
      if (!alive && wall_clock64() - born > kRelayGiveUpTicks) return;
      uint32_t ctr = raw - c.counter_base;
      if (threadIdx.x == 0)
        __hip_atomic_store(c.host_live, ctr < c.limit ? ctr : c.limit, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}

// Pause inside a long block while a preemption request stands.  Block-level preemption
// cannot act before the end of the running block; a block that lasts hundreds of
// microseconds (a 256x256 GEMM tile over a long K) would keep competing with the
// high-priority kernel for memory bandwidth and issue slots all that time.  Such a body
// calls this every few steps: the wave sleeps, holding its registers and LDS (the
// high-priority kernel runs beside it), until the request is withdrawn or `yield_ticks`
// have passed, so a high-priority kernel that does NOT fit beside it cannot deadlock.
struct YieldCtl {          // passed by value: taking the address of the kernel's control
  const uint32_t *flag;    // block would force it out of scalar registers into memory
  uint32_t epoch, ticks;
};
__device__ __forceinline__ void yield_while_preempted(const YieldCtl &y) {
  if (scalar_load_coherent(y.flag) != y.epoch) return;
  const unsigned long long t0 = wall_clock64();
  do {
    __builtin_amdgcn_s_sleep(64);
  } while (scalar_load_coherent(y.flag) == y.epoch &&
           wall_clock64() - t0 < (unsigned long long)y.ticks);
}

template <class Body>
__device__ __forceinline__ void ptb_body(const typename Body::Args &args, const PtbCtl &c) {
  __shared__ uint32_t s_idx[2];
  const uint32_t worker = blockIdx.x;
  // One lane reads flag and counter and broadcasts through LDS, so the exit decision is
  // uniform over the workgroup.  Order as in the paper: check the flag, then fetch; a
  // fetched index is always run.
  //
  // The word next to the flag says "grid exhausted": the worker whose fetch reaches the
  // end of the grid sets it, and the others then leave without one more fetch-add.  The
  // counter is one address that serves only ~88 M operations per second (loads included),
  // so W failing fetches at the very end would add W x 11 ns to every kernel.
  for (uint32_t it = 0;; ++it) {
    if (threadIdx.x == 0) {
      const unsigned long long f = __hip_atomic_load(
          reinterpret_cast<const unsigned long long *>(c.dev_flag), __ATOMIC_RELAXED,
          __HIP_MEMORY_SCOPE_AGENT);
      uint32_t first0 = kStop;
      if ((uint32_t)f != c.epoch && (uint32_t)(f >> 32) != c.epoch) {
        first0 = __hip_atomic_fetch_add(c.counter, c.chunk, __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_AGENT) - c.counter_base;
        if (first0 < c.limit && c.limit - first0 <= c.chunk)
          __hip_atomic_store(c.dev_flag + 1, c.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      s_idx[it & 1] = first0;
    }
    __syncthreads();
    const uint32_t first = s_idx[it & 1];
    if (first >= c.limit) break;  // uniform across the workgroup
    const uint32_t last = (c.limit - first < c.chunk) ? c.limit : first + c.chunk;
    for (uint32_t idx = first; idx < last; ++idx) {
      uint32_t bx, by, bz;
      delinearize(idx, c.gx, c.gy, bx, by, bz);
      if constexpr (Body::YIELDS)
        Body::run_yielding(args, bx, by, bz,
                           YieldCtl{c.flag_copies + (worker % kFlagCopies) * kFlagCopyStride, c.epoch,
                                    c.flag_copies != nullptr ? c.yield_ticks : 0u});
      else
        Body::run(args, bx, by, bz);
      record(c.cover, idx, bx, by, bz, c.segment, worker);
      // the paper ends every iteration with a barrier so that a worker handles one block
      // at a time; a body whose waves share no state across blocks does not need it
      if (Body::END_BARRIER) __syncthreads();
    }
  }
  // leave: the last worker of the segment publishes the progress to the host.
  // All of this is relaxed on purpose: an agent- or system-scope release here would make
  // every worker write back its whole L2 (tens of microseconds with a dirty output
  // tile).  Ordering comes from data dependence instead: a worker adds to `exited` only
  // after its last counter fetch has returned, so when the last worker sees the target
  // every other fetch has been performed, and it reads the counter after that.  Kernel
  // outputs become visible to the host at the end of the kernel as usual; the status
  // word only says that the workers are gone.
  if (threadIdx.x == 0) {
    uint32_t old = __hip_atomic_fetch_add(c.exited, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == c.exit_target) {
      uint32_t raw = __hip_atomic_load(c.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      uint32_t ctr = raw - c.counter_base;
      uint32_t progress = ctr < c.limit ? ctr : c.limit;
      __hip_atomic_store(c.host_raw, raw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      __hip_atomic_store(c.host_live, progress, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // both acknowledged before the status
      __hip_atomic_store(c.host_status, ((unsigned long long)c.epoch << 32) | progress,
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}
template <class Body>
__global__ __launch_bounds__(Body::THREADS, Body::MIN_WAVES) void ptb_kernel(typename Body::Args args, PtbCtl c) {
  ptb_body<Body>(args, c);
}

// Marker: stores a value into a pinned host word once earlier work on the stream is done.
__global__ void marker_kernel(uint32_t *word, uint32_t value) {
  if (threadIdx.x == 0)
    __hip_atomic_store(word, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ void set_word_kernel(uint32_t *word, uint32_t value) {
  if (threadIdx.x == 0)
    __hip_atomic_store(word, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace tally
