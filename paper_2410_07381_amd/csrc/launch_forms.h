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
//   static constexpr bool RANGE;             true if the body offers run_range(args, first,
//                                            last) for consecutive blocks of a 1-D grid
//   static __device__ void run(const Args&, uint32_t bx, uint32_t by, uint32_t bz);
//   static __device__ void run_be(const Args&, uint32_t bx, uint32_t by, uint32_t bz);
// run() performs the work of original block (bx,by,bz); run_be() is the same work as the
// best-effort forms (sliced, persistent workers) do it: identical arithmetic, but data that
// is touched once goes through non-temporal accesses so that it does not evict the
// high-priority job's data from the caches; every thread of the workgroup
// calls it and returns from it (no early exit), so the workgroup-wide barriers of the
// persistent-worker loop are reached by all threads (Section 4.1: divergent barriers
// stall a kernel for ever; hand-written bodies handle ragged tails by predication).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tally.h"

namespace tally {

// A preemption request is folded into the task counter by adding this to it: every later
// fetch then returns an index beyond any grid (grids have fewer than 2^30 blocks).
constexpr uint32_t kPreemptStep = 0x80000000u;
// Bit of the host's request word that says "do not pause inside blocks".
constexpr uint32_t kNoPauseBit = 0x80000000u;

// Device-side control block of one persistent-worker launch segment.
struct PtbCtl {
  uint32_t *counter;        // device: THE shared word.  Next task index (+ counter_base), plus
                            // kPreemptStep once a preemption request has been folded in.  It is
                            // never reset and wraps; indices are differences modulo 2^32.
  uint32_t *exited;         // device: workers that have exited, summed over all segments
  unsigned long long *pre;  // device: (epoch << 32 | progress) written by the relay right after
                            // it folded a request in: what its fetch-and-add returned
  const uint32_t *host_flag;  // pinned host memory: epoch the host wants preempted (| kNoPauseBit)
  unsigned long long *host_status;  // pinned: (epoch << 32 | progress) once drained
  uint32_t *host_live;      // pinned: progress mirrored while running
  uint32_t *host_raw;       // pinned: raw counter value at the drain (written before status)
  unsigned long long *host_relay;   // pinned: (epoch << 32 | raw counter) when the relay has ended
  uint32_t *host_relay_flags;       // pinned: bit 0 the relay gave up early, bit 1 it folded a request in
  tally_cover_rec *cover;   // device, may be null
  uint32_t total;           // logical blocks in the grid
  uint32_t limit;           // workers treat this as the end of the grid (== total normally)
  uint32_t epoch;           // id of this launch segment, unique for the life of the slot
  uint32_t exit_target;     // value of *exited after the last worker of this segment leaves
  uint32_t counter_base;    // raw counter value that stands for task index 0 of this job
  uint32_t workers;
  uint32_t chunk;           // task indices per fetch
  uint32_t single_pass;     // the workers' first fetches cover every index left: none fetches twice
  uint32_t segment;         // 0-based segment number, for the coverage records
  uint32_t gx, gy;          // logical grid extents (x fastest)
  uint32_t yield_ticks;     // longest pause inside ONE block, in 10 ns wall-clock ticks (0: never)
  uint32_t yield_mask;      // a pausing body looks at the pause word every (yield_mask + 1) steps
  uint32_t *flag_copies;    // device: kFlagCopies copies of the pause request (the epoch while
                            // workers are to pause inside their blocks, else 0), 128 B apart, for
                            // the mid-block polls (one address serves only ~80 M coherent scalar
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
  Body::run_be(args, bx, by, bz);
  record(ctl.cover, idx, bx, by, bz, ctl.segment, blockIdx.x);
}
template <class Body>
__global__ __launch_bounds__(Body::THREADS, Body::MIN_WAVES) void sliced_kernel(typename Body::Args args,
                                                               SliceCtl ctl) {
  sliced_body<Body>(args, ctl);
}

// ---- persistent-worker form (Section 4.1, preemption) --------------------------------
// The paper's worker reads a flag, then fetches and increments the task counter: two
// dependent round trips to memory per iteration.  Here the flag lives in the counter: a
// request is raised by adding 2^31 to it, a worker does ONE fetch-and-add per iteration
// and leaves when the index it got is beyond the grid, whether the grid is exhausted or a
// request was folded in.  A fetched index is always run (check and fetch are one
// operation, so the order question does not arise).
//
// The host raises a request with one store to pinned host memory (cheap to write, but a
// load from it crosses PCIe, far too slow for hundreds of workers to poll).  A one-wave
// relay kernel, launched just before the workers on a stream of its own, polls that word;
// when it names this segment the relay folds the request into the counter (its
// fetch-and-add returns the exact progress, which it leaves in `pre` for the last worker
// to publish) and, unless the request says otherwise, raises the pause word that workers
// inside long blocks poll.  It mirrors the progress to the host and leaves when every
// worker of the segment has exited, so its lifetime is bounded by the workers', which
// depend on nothing.
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
  uint32_t last = 0u;        // the host's word is 0 while nothing is asked
  bool added = false, gave_up = false;
  // The relay is launched before its workers.  Where the two cannot run side by side
  // (kernels executed strictly one after another) the workers cannot start until the
  // relay has ended: it leaves when neither the task counter nor the exit counter has
  // moved (by anyone but itself) for 20 ms; a request it folded in before that stands,
  // and the workers then find it when they start.
  const unsigned long long born = wall_clock64();
  uint32_t ctr0 = scalar_load_coherent(c.counter);
  const uint32_t gone0 = scalar_load_coherent(c.exited);
  bool alive = false;
  for (uint32_t n = 0;; ++n) {
    // once the request is in the counter only its withdrawal (the end of a pause) is news
    // from the host, and the exit counter is what matters: look at the host less often
    if (!added || (n & 3u) == 0u) {
      const uint32_t want = scalar_load_coherent(c.host_flag);
      if (want != last) {
        const bool mine = (want & ~kNoPauseBit) == c.epoch;
        if (mine && !added) {
          uint32_t p = 0;
          if (threadIdx.x == 0) {
            const uint32_t old = __hip_atomic_fetch_add(c.counter, kPreemptStep, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
            p = old - c.counter_base;
            p = p < c.limit ? p : c.limit;
            __hip_atomic_store(c.pre, ((unsigned long long)c.epoch << 32) | p, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(c.host_live, p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          }
          added = true;
          ctr0 += kPreemptStep;
        }
        // pause word: this segment's epoch while its workers are to pause inside blocks
        const uint32_t pause = (mine && !(want & kNoPauseBit)) ? c.epoch : 0u;
        if (c.flag_copies != nullptr && threadIdx.x < kFlagCopies)
          __hip_atomic_store(c.flag_copies + threadIdx.x * kFlagCopyStride, pause, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        last = want;
      }
    }
    // the counters of a slot only ever grow (they are never reset), so a relay that
    // starts late, even after its workers are long gone, still sees the target passed
    uint32_t gone = scalar_load_coherent(c.exited);
    if ((n & 255u) == 255u)  // and, now and then, through the path the workers' atomics use
      gone = __hip_atomic_load(c.exited, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((int32_t)(gone - c.exit_target) >= 0) break;
    if ((n & 15u) == 0u) {
      const uint32_t raw = scalar_load_coherent(c.counter);
      if (raw != ctr0 || gone != gone0) alive = true;
      if (!alive && wall_clock64() - born > kRelayGiveUpTicks) { gave_up = true; break; }
      if (!added) {
        const uint32_t ctr = raw - c.counter_base;
        if (threadIdx.x == 0)
          __hip_atomic_store(c.host_live, ctr < c.limit ? ctr : c.limit, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
  }
  // Last act: tell the host that this relay will not touch the counter any more, and what
  // the counter holds now (every worker has exited unless the relay gave up, in which case
  // the last worker's own report is the final one).
  if (threadIdx.x == 0) {
    const uint32_t raw = __hip_atomic_load(c.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(c.host_relay_flags, (gave_up ? 1u : 0u) | (added ? 2u : 0u), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __hip_atomic_store(c.host_relay, ((unsigned long long)c.epoch << 32) | raw, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

// Pause inside a long block while a preemption request stands.  Block-level preemption
// cannot act before the end of the running block; a block that lasts hundreds of
// microseconds (a 256x256 GEMM tile over a long K) would keep competing with the
// high-priority kernel for memory bandwidth and issue slots all that time.  Such a body
// calls this every few steps: the wave sleeps, holding its registers and LDS (the
// high-priority kernel runs beside it), until the request is withdrawn or the block's
// pause budget is spent, so a high-priority kernel that does NOT fit beside it cannot
// deadlock.  The budget is per block: `left` carries what remains of it across the polls.
struct YieldCtl {          // passed by value: taking the address of the kernel's control
  const uint32_t *flag;    // block would force it out of scalar registers into memory
  uint32_t epoch, ticks;
  uint32_t mask;           // poll when (step & mask) == mask
};
__device__ __forceinline__ void yield_while_preempted(const YieldCtl &y, uint32_t &left) {
  if (left == 0u || scalar_load_coherent(y.flag) != y.epoch) return;
  const unsigned long long t0 = wall_clock64();
  unsigned long long spent;
  do {
    __builtin_amdgcn_s_sleep(64);
    spent = wall_clock64() - t0;
  } while (scalar_load_coherent(y.flag) == y.epoch && spent < (unsigned long long)left);
  left = spent < (unsigned long long)left ? left - (uint32_t)spent : 0u;
}

constexpr uint32_t kPreSpinCap = 1u << 22;   // polls of `pre` before the last worker reports failure
constexpr uint32_t kProgressLost = 0xFFFFFFFFu;

template <class Body>
__device__ __forceinline__ void ptb_body(const typename Body::Args &args, const PtbCtl &c) {
  __shared__ uint32_t s_idx[2];
  const uint32_t worker = blockIdx.x;
  // One lane fetches and broadcasts through LDS, so the exit decision is uniform over the
  // workgroup.  An index at or beyond `limit` means: grid exhausted, or a request folded
  // into the counter; either way the worker leaves, and what it fetched before is done.
  for (uint32_t it = 0;; ++it) {
    if (threadIdx.x == 0)
      s_idx[it & 1] = __hip_atomic_fetch_add(c.counter, c.chunk, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT) - c.counter_base;
    __syncthreads();
    const uint32_t first = s_idx[it & 1];
    if (first >= c.limit) break;  // uniform across the workgroup
    const uint32_t last = (c.limit - first < c.chunk) ? c.limit : first + c.chunk;
    if constexpr (Body::RANGE) {
      // the blocks a fetch brought, handed to the body together (one-dimensional grids)
      if (last - first > 1) {
        Body::run_range(args, first, last);
        for (uint32_t idx = first; idx < last; ++idx) record(c.cover, idx, idx, 0, 0, c.segment, worker);
        if (c.single_pass) break;
        continue;
      }
    }
    for (uint32_t idx = first; idx < last; ++idx) {
      uint32_t bx, by, bz;
      delinearize(idx, c.gx, c.gy, bx, by, bz);
      if constexpr (Body::YIELDS)
        Body::run_yielding(args, bx, by, bz,
                           YieldCtl{c.flag_copies + (worker % kFlagCopies) * kFlagCopyStride, c.epoch,
                                    c.flag_copies != nullptr ? c.yield_ticks : 0u, c.yield_mask});
      else
        Body::run_be(args, bx, by, bz);
      record(c.cover, idx, bx, by, bz, c.segment, worker);
      // the paper ends every iteration with a barrier so that a worker handles one block
      // at a time; a body whose waves share no state across blocks does not need it
      if (Body::END_BARRIER) __syncthreads();
    }
    // the first fetches of all workers cover what is left: a second one could only fail
    if (c.single_pass) break;
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
      const uint32_t raw = __hip_atomic_load(c.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t ctr = raw - c.counter_base;
      uint32_t progress = ctr < c.limit ? ctr : c.limit;
      if (ctr & kPreemptStep) {
        // a request was folded in: the progress is what the relay's fetch-and-add returned.
        // The relay stores it right after that fetch-and-add, which has been performed
        // (its effect is in the counter), so this wait is short and ends whatever the
        // relay does next; the cap is a backstop that reports failure instead of hanging.
        progress = kProgressLost;
        for (uint32_t spin = 0; spin < kPreSpinCap; ++spin) {
          const unsigned long long pre =
              __hip_atomic_load(c.pre, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if ((uint32_t)(pre >> 32) == c.epoch) { progress = (uint32_t)pre; break; }
          __builtin_amdgcn_s_sleep(2);
        }
      }
      __hip_atomic_store(c.host_raw, raw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      if (progress != kProgressLost)
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

// One idle wave that stays on the GPU for `ticks` of the 100 MHz clock and then leaves
// (what a stream is kept busy with while its effect on another stream is measured).
__global__ void hold_kernel(uint32_t ticks) {
  const unsigned long long t0 = wall_clock64();
  while (wall_clock64() - t0 < (unsigned long long)ticks) __builtin_amdgcn_s_sleep(32);
}

__global__ void set_word_kernel(uint32_t *word, uint32_t value) {
  if (threadIdx.x == 0)
    __hip_atomic_store(word, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace tally
