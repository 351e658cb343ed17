// C ABI of the block-level kernel scheduling library (see include/tally.h).
//
// Host side of: native / sliced / persistent-worker launches (Section 4.1), preempt /
// drain / resume (Section 4.1), profile-guided configuration choice (Section 4.2, Eq. 1)
// and the two-stream priority scheduling loop (Section 4.2, Figure 4).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <map>
#include <mutex>
#include <new>
#include <thread>
#include <tuple>
#include <vector>

#include "../../include/tally.h"
#include "kernels_attn.h"
#include "kernels_gemm.h"
#include "kernels_stream.h"
#include "launch_forms.h"

using namespace tally;

namespace {

thread_local int g_last_hip = 0;
#define HIPCHK(expr)                                \
  do {                                              \
    hipError_t e_ = (expr);                         \
    if (e_ != hipSuccess) {                         \
      g_last_hip = (int)e_;                         \
      return TALLY_ERR_HIP;                         \
    }                                               \
  } while (0)

double now_us() {
  return std::chrono::duration<double, std::micro>(
             std::chrono::steady_clock::now().time_since_epoch())
      .count();
}

uint32_t cdiv(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---------------------------------------------------------------------------- registry
struct KernelOps {
  const char *name;
  size_t args_size;
  bool transformable;  // false: native form only
  int (*grid)(const void *args, tally_dim3 *g, tally_dim3 *b);
  hipError_t (*native)(hipStream_t, const void *args, tally_dim3 g, uint32_t urgent);
  hipError_t (*sliced)(hipStream_t, const void *args, uint32_t nblocks, const SliceCtl &);
  hipError_t (*ptb)(hipStream_t, const void *args, const PtbCtl &);
  hipError_t (*init)();
  int (*occupancy)(int *blocks_per_cu);
  // share of one logical block between two points at which a preempted worker pauses
  // (1 for bodies that only stop at block boundaries)
  double (*pause_fraction)(const void *args, uint32_t every);
  // what one workgroup of the persistent-worker kernel occupies on a compute unit
  hipError_t (*footprint)(uint32_t *lds_bytes, uint32_t *waves, uint32_t *regs_per_lane);
  // the same for one workgroup of the kernel in its original form
  hipError_t (*footprint_native)(uint32_t *lds_bytes, uint32_t *waves, uint32_t *regs_per_lane);
};

template <class Body>
hipError_t launch_native_t(hipStream_t s, const void *args, tally_dim3 g, uint32_t urgent) {
  typename Body::Args a;
  memcpy(&a, args, sizeof(a));
  hipLaunchKernelGGL(native_kernel<Body>, dim3(g.x, g.y, g.z), dim3(Body::THREADS), Body::DYN_LDS,
                     s, a, urgent);
  return hipGetLastError();
}
template <class Body>
hipError_t launch_sliced_t(hipStream_t s, const void *args, uint32_t nblocks, const SliceCtl &c) {
  typename Body::Args a;
  memcpy(&a, args, sizeof(a));
  hipLaunchKernelGGL(sliced_kernel<Body>, dim3(nblocks), dim3(Body::THREADS), Body::DYN_LDS, s, a,
                     c);
  return hipGetLastError();
}
template <class Body>
hipError_t launch_ptb_t(hipStream_t s, const void *args, const PtbCtl &c) {
  typename Body::Args a;
  memcpy(&a, args, sizeof(a));
  hipLaunchKernelGGL(ptb_kernel<Body>, dim3(c.workers), dim3(Body::THREADS), Body::DYN_LDS, s,
                     a, c);
  return hipGetLastError();
}
template <class Body>
hipError_t init_t() {
  if (Body::DYN_LDS > 64 * 1024) {
    hipError_t e;
    e = hipFuncSetAttribute((const void *)native_kernel<Body>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, Body::DYN_LDS);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)sliced_kernel<Body>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, Body::DYN_LDS);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)ptb_kernel<Body>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, Body::DYN_LDS);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
template <class Body>
int occupancy_t(int *blocks_per_cu) {
  HIPCHK(hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, ptb_kernel<Body>,
                                                      Body::THREADS, Body::DYN_LDS));
  return TALLY_OK;
}

template <class Body>
hipError_t footprint_t(uint32_t *lds_bytes, uint32_t *waves, uint32_t *regs_per_lane) {
  hipFuncAttributes attr;
  hipError_t e = hipFuncGetAttributes(&attr, (const void *)ptb_kernel<Body>);
  if (e != hipSuccess) return e;
  *lds_bytes = (uint32_t)attr.sharedSizeBytes + Body::DYN_LDS;
  *waves = Body::THREADS / 64;
  *regs_per_lane = ((uint32_t)attr.numRegs + 7u) & ~7u;
  return hipSuccess;
}

template <class Body>
hipError_t footprint_native_t(uint32_t *lds_bytes, uint32_t *waves, uint32_t *regs_per_lane) {
  hipFuncAttributes attr;
  hipError_t e = hipFuncGetAttributes(&attr, (const void *)native_kernel<Body>);
  if (e != hipSuccess) return e;
  *lds_bytes = (uint32_t)attr.sharedSizeBytes + Body::DYN_LDS;
  *waves = Body::THREADS / 64;
  *regs_per_lane = ((uint32_t)attr.numRegs + 7u) & ~7u;
  return hipSuccess;
}
hipError_t footprint_attn(uint32_t *lds_bytes, uint32_t *waves, uint32_t *regs_per_lane) {
  hipFuncAttributes attr;
  hipError_t e = hipFuncGetAttributes(&attr, (const void *)attn_decode_partial);
  if (e != hipSuccess) return e;
  *lds_bytes = (uint32_t)attr.sharedSizeBytes;
  *waves = 4;
  *regs_per_lane = ((uint32_t)attr.numRegs + 7u) & ~7u;
  return hipSuccess;
}

// Row kernels in their original form: rows that fit the narrow instantiation get the kernel
// that needs a quarter of the registers.
template <class Wide, class Narrow>
hipError_t launch_native_rows_t(hipStream_t s, const void *args, tally_dim3 g, uint32_t urgent) {
  typename Wide::Args a;
  memcpy(&a, args, sizeof(a));
  if (a.cols <= Narrow::MAX_COLS) return launch_native_t<Narrow>(s, args, g, urgent);
  return launch_native_t<Wide>(s, args, g, urgent);
}

const tally_dim3 kBlock256 = {256, 1, 1};

int grid_saxpy(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_saxpy_args *>(p);
  if (!a->x || !a->y || a->n == 0) return TALLY_ERR_INVALID_ARG;
  *g = {cdiv(a->n, 256), 1, 1};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_reduce_sum(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_reduce_sum_args *>(p);
  if (!a->x || !a->partial || a->n == 0 || !aligned16(a->x)) return TALLY_ERR_INVALID_ARG;
  if (a->n > 4096ull * 0x7FFFFFFFull) return TALLY_ERR_INVALID_ARG;
  *g = {cdiv(a->n, 4096), 1, 1};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_reduce_final(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_reduce_final_args *>(p);
  if (!a->partial || !a->total || a->count == 0) return TALLY_ERR_INVALID_ARG;
  *g = {1, 1, 1};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_gemm_common(const tally_gemm_bf16_args *a) {
  if (!a->A || !a->Bt || !a->C || !a->m || !a->n || !a->k || !a->batch) return TALLY_ERR_INVALID_ARG;
  if (!aligned16(a->A) || !aligned16(a->Bt) || (a->stride_a % 8) || (a->stride_b % 8))
    return TALLY_ERR_INVALID_ARG;
  if ((a->lda && (a->lda < a->k || (a->lda % 8))) || (a->ldb && (a->ldb < a->k || (a->ldb % 8))))
    return TALLY_ERR_INVALID_ARG;
  const uint64_t lda = a->lda ? a->lda : a->k, ldb = a->ldb ? a->ldb : a->k;
  if (lda > (1u << 20) || ldb > (1u << 20)) return TALLY_ERR_INVALID_ARG;  // 32-bit byte offsets per tile
  if (a->batch > 1 && (a->stride_a < (uint64_t)(a->m - 1) * lda + a->k ||
                       a->stride_b < (uint64_t)(a->n - 1) * ldb + a->k ||
                       a->stride_c < (uint64_t)a->m * a->n))
    return TALLY_ERR_INVALID_ARG;
  return TALLY_OK;
}
int grid_gemm(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_gemm_bf16_args *>(p);
  int rc = grid_gemm_common(a);
  if (rc) return rc;
  if ((a->m % 256) || (a->n % 256) || (a->k % 32)) return TALLY_ERR_INVALID_ARG;
  if (!aligned16(a->C) || (a->stride_c % 8)) return TALLY_ERR_INVALID_ARG;  // 16-byte stores
  *g = {a->n / 256, a->m / 256, a->batch};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_gemm_n128(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_gemm_bf16_args *>(p);
  int rc = grid_gemm_common(a);
  if (rc) return rc;
  if ((a->m % 256) || (a->n % 128) || (a->k % 32)) return TALLY_ERR_INVALID_ARG;
  if (!aligned16(a->C) || (a->stride_c % 8)) return TALLY_ERR_INVALID_ARG;  // 16-byte stores
  *g = {a->n / 128, a->m / 256, a->batch};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_gemm_small(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_gemm_bf16_args *>(p);
  int rc = grid_gemm_common(a);
  if (rc) return rc;
  if (a->k % 32) return TALLY_ERR_INVALID_ARG;
  *g = {cdiv(a->n, 32), cdiv(a->m, 32), a->batch};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_gemv(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_gemv_bf16_args *>(p);
  if (!a->x || !a->W || !a->y || !a->n || !a->k || (a->k % 8) || !aligned16(a->x) || !aligned16(a->W))
    return TALLY_ERR_INVALID_ARG;
  *g = {cdiv(a->n, 4), 1, 1};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_softmax(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_softmax_f32_args *>(p);
  if (!a->x || !a->y || !a->rows || !a->cols || (a->cols % 4) || a->cols > 8192 || !aligned16(a->x) ||
      !aligned16(a->y))
    return TALLY_ERR_INVALID_ARG;
  *g = {cdiv(a->rows, 4), 1, 1};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_layernorm(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_layernorm_f32_args *>(p);
  if (!a->x || !a->y || !a->gamma || !a->beta || !a->rows || !a->cols || (a->cols % 4) ||
      a->cols > 8192 || !aligned16(a->x) || !aligned16(a->y) || !aligned16(a->gamma) ||
      !aligned16(a->beta))
    return TALLY_ERR_INVALID_ARG;
  *g = {cdiv(a->rows, 4), 1, 1};
  *b = kBlock256;
  return TALLY_OK;
}
int grid_attn(const void *p, tally_dim3 *g, tally_dim3 *b) {
  auto *a = static_cast<const tally_attn_decode_args *>(p);
  if (!a->q || !a->K || !a->V || !a->out || !a->scratch || !a->tokens || !a->heads || a->dim != 128 ||
      a->tokens > kAttnSplits * kAttnMaxChunk ||
      !aligned16(a->q) || !aligned16(a->K) || !aligned16(a->V))
    return TALLY_ERR_INVALID_ARG;
  *g = {a->heads, 1, 1};
  *b = kBlock256;
  return TALLY_OK;
}

template <class Body>
double pause_fraction_t(const void *args, uint32_t every) {
  if constexpr (Body::YIELDS) {
    typename Body::Args a;
    memcpy(&a, args, sizeof(a));
    return Body::pause_fraction(a, every);
  } else {
    return 1.0;
  }
}

#define OPS(Body, nm, gridfn)                                                              \
  {nm, sizeof(Body::Args), true, gridfn, launch_native_t<Body>, launch_sliced_t<Body>,     \
   launch_ptb_t<Body>, init_t<Body>, occupancy_t<Body>, pause_fraction_t<Body>,              \
   footprint_t<Body>, footprint_native_t<Body>}

const KernelOps kOps[TALLY_K_COUNT] = {
    OPS(SaxpyBody, "saxpy", grid_saxpy),
    OPS(ReduceSumBody, "reduce_sum", grid_reduce_sum),
    OPS(ReduceFinalBody, "reduce_final", grid_reduce_final),
    OPS(GemmBody, "gemm_bf16", grid_gemm),
    OPS(GemvBody, "gemv_bf16", grid_gemv),
    {"softmax_f32", sizeof(SoftmaxBody::Args), true, grid_softmax,
     launch_native_rows_t<SoftmaxBody, SoftmaxNarrowBody>, launch_sliced_t<SoftmaxBody>,
     launch_ptb_t<SoftmaxBody>, init_t<SoftmaxBody>, occupancy_t<SoftmaxBody>,
     pause_fraction_t<SoftmaxBody>, footprint_t<SoftmaxBody>, footprint_native_t<SoftmaxBody>},
    {"layernorm_f32", sizeof(LayerNormBody::Args), true, grid_layernorm,
     launch_native_rows_t<LayerNormBody, LayerNormNarrowBody>, launch_sliced_t<LayerNormBody>,
     launch_ptb_t<LayerNormBody>, init_t<LayerNormBody>, occupancy_t<LayerNormBody>,
     pause_fraction_t<LayerNormBody>, footprint_t<LayerNormBody>, footprint_native_t<LayerNormBody>},
    {"attn_decode_bf16", sizeof(tally_attn_decode_args), false, grid_attn, launch_attn_decode,
     nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, footprint_attn},
    OPS(GemmSmallBody, "gemm_bf16_small", grid_gemm_small),
    OPS(GemmN128Body, "gemm_bf16_n128", grid_gemm_n128),
};

constexpr size_t kMaxArgs = 96;
constexpr int kSlots = 64;
constexpr int kMaxShunned = 64;
constexpr int kMaxSide = 2 * 8 + 2;
constexpr int kMaxBeClients = 8;
constexpr size_t kDevSlotBytes = 512;   // counter | pre | exited, 128 B apart
constexpr size_t kHostSlotBytes = 256;  // host_flag | status,live,raw,relay,relay_flags | slice_done
constexpr size_t kCopySlotBytes = kFlagCopies * kFlagCopyStride * sizeof(uint32_t);

enum JobKind { KIND_PTB = 0, KIND_SLICED = 1, KIND_NATIVE = 2 };

// One kernel's profiling record.  Measurements are sums over real executions of the kernel
// (each invocation measures one candidate once); the configuration is fixed when every
// candidate has `runs` samples.
typedef std::tuple<uint32_t, uint32_t, uint32_t, uint32_t, uint32_t> ProfileKey;
struct ProfileEntry {
  std::vector<tally_config> cands;
  std::vector<double> sum_ms;
  std::vector<uint32_t> samples;
  int chosen = -1;
  double threshold_ms = 0.0;   // the threshold `chosen` was selected under
};

constexpr uint32_t kStaticAttnMaxHeads = TALLY_ATTN_STATIC_MAX_HEADS;
constexpr size_t kStaticAttnBytes =
    (size_t)kStaticAttnMaxHeads * kAttnSplits * kAttnRec * sizeof(float);

}  // namespace

// Split records of the decode-attention kernels for callers that may not allocate: device
// memory that belongs to the library's code object, one copy per GPU, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// address kernels receive is the one that call returns, kept per context.  (File scope,
// not an unnamed namespace: there the device symbol stays local to the code object and the
// runtime cannot look it up.)
static __device__ __align__(256) unsigned char static_scratch[kStaticAttnBytes];

struct tally_ctx {
  hipStream_t hi, be;
  hipStream_t ctl;           // owned: carries the relay kernels, default priority
  // streams that new jobs take (normally be / ctl); the scheduler points them at a
  // best-effort client's own pair while it launches for that client
  hipStream_t cur_be, cur_ctl;
  hipStream_t client_be[kMaxBeClients], client_ctl[kMaxBeClients];  // owned, [0] unused
  // streams that were created and found to delay the high-priority stream (same hardware
  // pipe): never used, kept until the context goes so that their queues stay taken
  hipStream_t shunned[kMaxShunned];
  int n_shunned;
  hipStream_t side[kMaxSide];   // the caller's best-effort stream and the streams chosen so far
  int n_side;
  bool side_crowded;            // a stream had to be taken although it delays the high-priority one
  uint32_t probe_seq;
  bool be_delays_hi;         // the caller's best-effort stream shares the high-priority one's pipe
  unsigned char *dev_pool;   // device
  uint32_t *copy_pool;       // device: per slot, kFlagCopies copies of the flag word
  unsigned char *host_pool;  // pinned host
  unsigned char *host_pool_dev;
  bool slot_used[kSlots];
  int next_slot;
  // device words of a slot are never reset: the host tracks their current values instead
  // (slot_counter: the raw task counter as the slot's last job left it)
  uint32_t slot_counter[kSlots], slot_exited[kSlots], slot_epoch[kSlots];
  uint32_t *marker_host;     // pinned: [0] hi, [32] be (separate lines)
  uint32_t *marker_dev;
  uint32_t num_cus;
  uint32_t lds_per_cu;
  uint32_t max_workers[TALLY_K_COUNT];  // persistent-worker workgroups resident at once, per kernel
  // what one workgroup occupies on a compute unit (LDS bytes, waves, registers per lane):
  // [0] persistent-worker form, [1] original form; asked of the runtime once, at creation
  uint32_t foot[TALLY_K_COUNT][2][3];
  uint32_t yield_ticks;      // bound of a mid-block pause, 10 ns ticks
  uint32_t yield_every;      // steps between two looks at the pause word (a power of two)
  void *static_attn_scratch; // this device's address of static_scratch
  int device;
  int live_jobs;
  // profile-guided configuration (Section 4.2): per (kernel, grid, block) the candidate
  // table with its measurements, and the choice once every candidate has been measured
  std::mutex profile_mu;
  std::map<ProfileKey, ProfileEntry> profiles;
};

struct tally_job {
  tally_ctx *ctx;
  hipStream_t be, ctl;       // the streams this job's kernels and relays go to
  const KernelOps *ops;
  alignas(16) unsigned char args[kMaxArgs];
  tally_dim3 grid;
  uint32_t total;
  int kind;
  int slot;
  tally_cover_rec *cover;
  std::atomic<int> state;
  std::atomic<uint32_t> progress;
  // persistent workers
  uint32_t workers, chunk, epoch, limit;
  uint32_t yield_ticks;      // the context's pause bound when the job was made
  uint32_t yield_every;
  uint32_t counter_base;     // raw counter value standing for task index 0
  uint32_t segments;         // launch segments so far
  bool relay_pending;        // a relay of this job may still be running (its report is not in)
  bool failed;               // the device could not report the progress of a preempted segment
  std::atomic<uint32_t> request_word;  // what was last stored in the host's request word
  // sliced
  uint32_t slice_blocks, max_in_flight, next_off, issued, retired, segment;
  std::atomic<bool> stop_issuing;
  // preemption latency
  std::atomic<double> t_preempt;
  double preempt_latency_us;

  uint32_t *d_counter() { return (uint32_t *)(ctx->dev_pool + slot * kDevSlotBytes); }
  unsigned long long *d_pre() { return (unsigned long long *)(ctx->dev_pool + slot * kDevSlotBytes + 128); }
  uint32_t *d_exited() { return (uint32_t *)(ctx->dev_pool + slot * kDevSlotBytes + 256); }
  unsigned char *h_base() { return ctx->host_pool + slot * kHostSlotBytes; }
  unsigned char *h_base_dev() { return ctx->host_pool_dev + slot * kHostSlotBytes; }
  uint32_t *h_flag() { return (uint32_t *)h_base(); }
  unsigned long long *h_status() { return (unsigned long long *)(h_base() + 64); }
  uint32_t *h_live() { return (uint32_t *)(h_base() + 72); }
  uint32_t *h_raw() { return (uint32_t *)(h_base() + 76); }
  unsigned long long *h_relay() { return (unsigned long long *)(h_base() + 80); }
  uint32_t *h_relay_flags() { return (uint32_t *)(h_base() + 88); }
  uint32_t *h_slice_done() { return (uint32_t *)(h_base() + 128); }
};

namespace {

int check_desc(const tally_kernel_desc *d, const KernelOps **ops_out, tally_dim3 *grid) {
  if (!d || !d->args || d->kernel_id >= TALLY_K_COUNT) return TALLY_ERR_INVALID_ARG;
  const KernelOps *ops = &kOps[d->kernel_id];
  if (d->args_size != ops->args_size || ops->args_size > kMaxArgs) return TALLY_ERR_INVALID_ARG;
  tally_dim3 g, b;
  int rc = ops->grid(d->args, &g, &b);
  if (rc) return rc;
  if (d->grid.x != g.x || d->grid.y != g.y || d->grid.z != g.z || d->block.x != b.x ||
      d->block.y != b.y || d->block.z != b.z)
    return TALLY_ERR_INVALID_ARG;
  // (task indices and a folded-in preemption request share one 32-bit word)
  if ((uint64_t)g.x * g.y * g.z > 0x40000000ull) return TALLY_ERR_INVALID_ARG;
  *ops_out = ops;
  *grid = g;
  return TALLY_OK;
}

int new_job(tally_ctx *ctx, const tally_kernel_desc *desc, int kind, int coverage, tally_job **out) {
  const KernelOps *ops;
  tally_dim3 g;
  int rc = check_desc(desc, &ops, &g);
  if (rc) return rc;
  if (kind != KIND_NATIVE && !ops->transformable) return TALLY_ERR_UNSUPPORTED;
  // slots are handed out round-robin so that a freed slot rests before it is reused
  int slot = -1;
  for (int i = 0; i < kSlots; ++i) {
    int s = (ctx->next_slot + i) % kSlots;
    if (!ctx->slot_used[s]) { slot = s; break; }
  }
  if (slot < 0) return TALLY_ERR_NOMEM;
  ctx->next_slot = (slot + 1) % kSlots;
  tally_job *j = new (std::nothrow) tally_job();
  if (!j) return TALLY_ERR_NOMEM;
  j->ctx = ctx;
  j->be = ctx->cur_be;
  j->ctl = ctx->cur_ctl;
  j->ops = ops;
  memcpy(j->args, desc->args, ops->args_size);
  j->grid = g;
  j->total = g.x * g.y * g.z;
  j->kind = kind;
  j->slot = slot;
  j->cover = nullptr;
  j->state = TALLY_JOB_QUEUED;
  j->progress = 0;
  j->workers = j->chunk = j->epoch = j->segments = 0;
  j->counter_base = ctx->slot_counter[slot];
  j->yield_ticks = ctx->yield_ticks;
  j->yield_every = ctx->yield_every;
  j->limit = j->total;
  j->relay_pending = false;
  j->failed = false;
  j->request_word = 0;
  j->slice_blocks = j->max_in_flight = j->next_off = j->issued = j->retired = j->segment = 0;
  j->stop_issuing = false;
  j->t_preempt = 0.0;
  j->preempt_latency_us = -1.0;
  hipError_t e = hipSuccess;
  if (coverage) {
    e = hipMalloc((void **)&j->cover, sizeof(tally_cover_rec) * (size_t)j->total);
    if (e == hipSuccess)
      e = hipMemsetAsync(j->cover, 0, sizeof(tally_cover_rec) * (size_t)j->total, j->be);
  }
  if (e != hipSuccess) {
    g_last_hip = (int)e;
    if (j->cover) (void)hipFree(j->cover);
    delete j;
    return e == hipErrorOutOfMemory ? TALLY_ERR_NOMEM : TALLY_ERR_HIP;
  }
  memset(j->h_base(), 0, kHostSlotBytes);
  ctx->slot_used[slot] = true;
  ctx->live_jobs++;
  *out = j;
  return TALLY_OK;
}

// The relay of the job's last segment reports when it has ended and what the counter then
// held.  Until that report is in, the relay may still fold a late request into the counter,
// so neither a new segment nor a new job may use the slot's counter.  The relay ends within
// microseconds of its workers (or after its 20 ms give-up bound when it ran before them).
int settle_relay(tally_job *j) {
  if (!j->relay_pending) return TALLY_OK;
  for (uint64_t spins = 1;; ++spins) {
    const unsigned long long r = __atomic_load_n(j->h_relay(), __ATOMIC_ACQUIRE);
    if ((uint32_t)(r >> 32) == j->epoch) {
      const uint32_t flags = __atomic_load_n(j->h_relay_flags(), __ATOMIC_RELAXED);
      // a relay that gave up ended before its workers: their own report has the final value
      const uint32_t raw = (flags & 1u) ? __atomic_load_n(j->h_raw(), __ATOMIC_RELAXED) : (uint32_t)r;
      j->ctx->slot_counter[j->slot] = raw;
      j->relay_pending = false;
      return TALLY_OK;
    }
    if ((spins & 0xFFFFFu) == 0) {
      hipError_t q = hipStreamQuery(j->ctl);
      if (q != hipSuccess && q != hipErrorNotReady) { g_last_hip = (int)q; return TALLY_ERR_HIP; }
    }
  }
}

// Launch the workers (and their relay) for task indices [progress, limit).  Requires the
// job's previous segment, if any, to have drained.
int ptb_launch_segment(tally_job *j, uint32_t limit) {
  tally_ctx *ctx = j->ctx;
  const int slot = j->slot;
  int rc = settle_relay(j);
  if (rc) return rc;
  const uint32_t start = j->progress.load();
  // The counter is never rewound: failed fetches of the last segment (after a request, or
  // beyond a stop_at limit) have advanced it, so the value that stands for task index 0
  // moves instead, such that the next index handed out is `start` again.
  j->counter_base = ctx->slot_counter[slot] - start;
  j->epoch = ctx->slot_epoch[slot] + 1;
  j->limit = limit < j->total ? limit : j->total;
  __atomic_store_n(j->h_flag(), 0u, __ATOMIC_RELEASE);   // no request stands against the new segment
  j->request_word = 0;
  PtbCtl c;
  c.counter = j->d_counter();
  c.exited = j->d_exited();
  c.pre = j->d_pre();
  c.host_flag = (const uint32_t *)j->h_base_dev();
  c.host_status = (unsigned long long *)(j->h_base_dev() + 64);
  c.host_live = (uint32_t *)(j->h_base_dev() + 72);
  c.host_raw = (uint32_t *)(j->h_base_dev() + 76);
  c.host_relay = (unsigned long long *)(j->h_base_dev() + 80);
  c.host_relay_flags = (uint32_t *)(j->h_base_dev() + 88);
  c.cover = j->cover;
  c.total = j->total;
  c.limit = j->limit;
  c.epoch = j->epoch;
  c.exit_target = ctx->slot_exited[slot] + j->workers;
  c.counter_base = j->counter_base;
  c.workers = j->workers;
  c.chunk = j->chunk;
  c.single_pass = (j->limit > start ? (uint64_t)(j->limit - start) : 0ull) <=
                          (uint64_t)j->chunk * j->workers ? 1u : 0u;
  c.segment = j->segments;
  c.gx = j->grid.x;
  c.gy = j->grid.y;
  c.yield_ticks = j->yield_ticks;
  c.yield_mask = j->yield_every - 1;
  c.flag_copies = ctx->copy_pool + (size_t)slot * (kCopySlotBytes / sizeof(uint32_t));
  // The relay goes first, on its own stream: once the workers are on the GPU there may be
  // no wave slot or register left anywhere for it (four 128-register softmax workgroups
  // fill a compute unit exactly; one slot kept free was taken by whichever workgroup came
  // first), and without the relay a request is never seen.  Its exit depends only on the
  // slot's exit counter reaching the target, so it may start early; where kernels are run
  // strictly one at a time (counter collection under a profiler) it gives up when no
  // worker has shown up for a while, and a request raised after that goes unseen.
  hipLaunchKernelGGL(relay_kernel, dim3(1), dim3(64), 0, j->ctl, c);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {  // nothing was enqueued: the slot's bookkeeping is unchanged
    g_last_hip = (int)e;
    return TALLY_ERR_HIP;
  }
  j->relay_pending = true;
  e = j->ops->ptb(j->be, j->args, c);
  ctx->slot_epoch[slot] = j->epoch;
  ctx->slot_exited[slot] = c.exit_target;
  if (e != hipSuccess) {
    // no workers will ever count themselves out: do it for them, so that the relay ends
    g_last_hip = (int)e;
    hipLaunchKernelGGL(set_word_kernel, dim3(1), dim3(64), 0, j->be, j->d_exited(), c.exit_target);
    (void)hipGetLastError();
    return TALLY_ERR_HIP;
  }
  j->segments += 1;
  j->t_preempt = 0.0;
  j->state = TALLY_JOB_RUNNING;
  return TALLY_OK;
}

int sliced_issue(tally_job *j) {
  while (!j->stop_issuing.load() && j->next_off < j->total &&
         j->issued - j->retired < j->max_in_flight) {
    uint32_t n = j->total - j->next_off;
    if (n > j->slice_blocks) n = j->slice_blocks;
    SliceCtl c;
    c.cover = j->cover;
    c.offset = j->next_off;
    c.gx = j->grid.x;
    c.gy = j->grid.y;
    c.segment = j->segment;
    HIPCHK(j->ops->sliced(j->be, j->args, n, c));
    j->issued += 1;
    j->next_off += n;
    hipLaunchKernelGGL(marker_kernel, dim3(1), dim3(64), 0, j->be,
                       (uint32_t *)(j->h_base_dev() + 128), j->issued);
    HIPCHK(hipGetLastError());
  }
  return TALLY_OK;
}

// Bring the host-side state up to date with what the device has published.
void refresh(tally_job *j) {
  if (j->state.load() != TALLY_JOB_RUNNING) return;
  if (j->kind == KIND_PTB) {
    unsigned long long st = __atomic_load_n(j->h_status(), __ATOMIC_ACQUIRE);
    if ((uint32_t)(st >> 32) == j->epoch) {
      uint32_t p = (uint32_t)st;
      if (p == kProgressLost) {   // the device could not tell: keep the last known progress
        j->failed = true;
        p = j->progress.load();
      }
      j->progress = p;
      double tp = j->t_preempt.load();
      j->preempt_latency_us = (tp > 0.0 && p < j->total) ? now_us() - tp : -1.0;
      j->state = (p >= j->total) ? TALLY_JOB_COMPLETE : TALLY_JOB_STOPPED;
    } else {
      uint32_t live = __atomic_load_n(j->h_live(), __ATOMIC_RELAXED);
      if (live > j->progress.load()) j->progress = live;
    }
  } else {
    uint32_t done = __atomic_load_n(j->h_slice_done(), __ATOMIC_ACQUIRE);
    j->retired = done;
    if (j->kind == KIND_NATIVE) {
      if (done >= 1) { j->progress = j->total; j->state = TALLY_JOB_COMPLETE; }
      return;
    }
    uint64_t p = (uint64_t)done * j->slice_blocks;
    if (p > j->total) p = j->total;
    j->progress = (uint32_t)p;
    if (p >= j->total) {
      j->state = TALLY_JOB_COMPLETE;
    } else if (j->stop_issuing.load() && j->retired == j->issued) {
      double tp = j->t_preempt.load();
      j->preempt_latency_us = tp > 0.0 ? now_us() - tp : -1.0;
      j->state = TALLY_JOB_STOPPED;
    }
  }
}

int launch_be_item(tally_ctx *ctx, const tally_be_item *it, tally_job **out);

}  // namespace

// ================================================================================ C ABI
namespace {

// Do kernels resident on `other` and on the streams in `also`, all at once, delay kernels
// on the high-priority stream?  The GPU's command processors (one per die) serve the
// hardware queues through four pipes each, and HIP hands streams to hardware queues in the
// order of their first use.  Measured on this part, with one idle wave held per stream: a
// resident kernel on a queue that shares the high-priority queue's pipe delays the start
// of every high-priority kernel by 8 to 10 us (a 7 us request: 21 us instead of 11 us on the
// device); any number of resident kernels on the other pipes cost nothing.  The sharing can
// differ from die to die: with two best-effort clients one of the four streams in use
// delayed every high-priority kernel that had workgroups on all dies by 11 to 16 us and a
// one-workgroup kernel not at all, so the probe kernel below has workgroups on every die.
// (With GPU_MAX_HW_QUEUES at its default two streams may even be one queue and run one after
// the other.)  Persistent workers and their relays stay resident for a whole kernel, so the
// streams that carry them are chosen by this measurement, neither HIP nor the driver
// telling which queue a stream got: the shortest of a few round trips on the high-priority
// stream, first with everything idle, then with the streams held busy.
bool delays_hi_stream(tally_ctx *ctx, hipStream_t other, const hipStream_t *also, int n_also) {
  uint32_t *word_dev = ctx->marker_dev + 16, *word_host = ctx->marker_host + 16;
  auto round_trip_us = [&](int reps) {
    double best = 1e30;
    for (int i = 0; i < reps; ++i) {
      const uint32_t v = ++ctx->probe_seq;
      const double t0 = now_us();
      // a kernel with workgroups on every die, then the marker: a one-workgroup kernel alone
      // does not feel every conflict (each die's command processor serves its own share)
      hipLaunchKernelGGL(hold_kernel, dim3(64), dim3(64), 0, ctx->hi, 1u);
      hipLaunchKernelGGL(marker_kernel, dim3(1), dim3(64), 0, ctx->hi, word_dev, v);
      if (hipGetLastError() != hipSuccess) return 0.0;
      while (__atomic_load_n(word_host, __ATOMIC_ACQUIRE) != v && now_us() - t0 < 2.0e5) {}
      const double dt = now_us() - t0;
      if (dt < best) best = dt;
    }
    return best;
  };
  auto sync_all = [&]() {
    bool ok = hipStreamSynchronize(ctx->hi) == hipSuccess && hipStreamSynchronize(other) == hipSuccess;
    for (int i = 0; i < n_also; ++i) ok = (hipStreamSynchronize(also[i]) == hipSuccess) && ok;
    return ok;
  };
  // a stream gets its hardware queue with its first kernel, which takes a millisecond:
  // let that happen before anything is timed
  hipLaunchKernelGGL(hold_kernel, dim3(1), dim3(64), 0, other, 1u);
  if (hipGetLastError() != hipSuccess || !sync_all()) return false;
  const double idle = round_trip_us(8);
  for (int i = 0; i <= n_also; ++i) {
    hipLaunchKernelGGL(hold_kernel, dim3(1), dim3(64), 0, i < n_also ? also[i] : other, 60000u);   // 600 us
    if (hipGetLastError() != hipSuccess) { (void)sync_all(); return false; }
  }
  const double t0 = now_us();
  while (now_us() - t0 < 40.0) {}                       // let them start
  const double busy = round_trip_us(8);
  (void)sync_all();
  if (getenv("TALLY_DEBUG_STREAMS"))
    fprintf(stderr, "[tally] stream %p beside %d others: marker round trip %.1f us idle, %.1f us busy\n",
            (void *)other, n_also, idle, busy);
  return busy > idle + 4.0;
}

// A new stream for resident best-effort work (workers, relays) that, busy together with
// the streams already chosen for such work, does not delay the high-priority stream.
// Streams that do are set aside.  Four pipes: after four candidates in a row that do, there
// is no better one to be had (more resident queues than free pipes) and the last is taken.
hipError_t make_side_stream(tally_ctx *ctx, hipStream_t *out) {
  for (int tries = 0;; ++tries) {
    hipStream_t s;
    hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);
    if (e != hipSuccess) return e;
    const bool delays = delays_hi_stream(ctx, s, ctx->side, ctx->n_side);
    if (!delays || tries >= 3 || ctx->n_shunned >= kMaxShunned) {
      if (delays) ctx->side_crowded = true;
      if (ctx->n_side < kMaxSide) ctx->side[ctx->n_side++] = s;
      *out = s;
      return hipSuccess;
    }
    ctx->shunned[ctx->n_shunned++] = s;
  }
}

}  // namespace

extern "C" {

int tally_create(tally_ctx **out, void *hip_stream_hi, void *hip_stream_be) {
  if (!out) return TALLY_ERR_INVALID_ARG;
  tally_ctx *c = new (std::nothrow) tally_ctx();
  if (!c) return TALLY_ERR_NOMEM;
  c->hi = (hipStream_t)hip_stream_hi;
  c->be = (hipStream_t)hip_stream_be;
  c->ctl = nullptr;
  memset(c->client_be, 0, sizeof(c->client_be));
  memset(c->client_ctl, 0, sizeof(c->client_ctl));
  c->dev_pool = nullptr;
  c->copy_pool = nullptr;
  c->host_pool = nullptr;
  c->marker_host = nullptr;
  c->static_attn_scratch = nullptr;
  memset(c->slot_used, 0, sizeof(c->slot_used));
  memset(c->slot_counter, 0, sizeof(c->slot_counter));
  memset(c->slot_exited, 0, sizeof(c->slot_exited));
  memset(c->slot_epoch, 0, sizeof(c->slot_epoch));
  c->live_jobs = 0;
  c->next_slot = 0;
  c->n_shunned = 0;
  c->n_side = 0;
  c->side_crowded = false;
  c->probe_seq = 0;
  c->ctl = nullptr;
  hipError_t e;
  int dev = 0;
  hipDeviceProp_t prop;
  if ((e = hipGetDevice(&dev)) != hipSuccess || (e = hipGetDeviceProperties(&prop, dev)) != hipSuccess ||
      (e = hipMalloc((void **)&c->dev_pool, kSlots * kDevSlotBytes)) != hipSuccess ||
      (e = hipMemset(c->dev_pool, 0, kSlots * kDevSlotBytes)) != hipSuccess ||
      (e = hipMalloc((void **)&c->copy_pool, kSlots * kCopySlotBytes)) != hipSuccess ||
      (e = hipMemset(c->copy_pool, 0, kSlots * kCopySlotBytes)) != hipSuccess ||
      (e = hipHostMalloc((void **)&c->host_pool, kSlots * kHostSlotBytes, hipHostMallocDefault)) != hipSuccess ||
      (e = hipHostGetDevicePointer((void **)&c->host_pool_dev, c->host_pool, 0)) != hipSuccess ||
      (e = hipGetSymbolAddress(&c->static_attn_scratch, HIP_SYMBOL(static_scratch))) != hipSuccess ||
      (e = hipHostMalloc((void **)&c->marker_host, 256, hipHostMallocDefault)) != hipSuccess ||
      (e = hipHostGetDevicePointer((void **)&c->marker_dev, c->marker_host, 0)) != hipSuccess) {
    g_last_hip = (int)e;
    if (c->ctl) (void)hipStreamDestroy(c->ctl);
    if (c->dev_pool) (void)hipFree(c->dev_pool);
    if (c->copy_pool) (void)hipFree(c->copy_pool);
    if (c->host_pool) (void)hipHostFree(c->host_pool);
    if (c->marker_host) (void)hipHostFree(c->marker_host);
    delete c;
    return TALLY_ERR_HIP;
  }
  memset(c->host_pool, 0, kSlots * kHostSlotBytes);
  memset(c->marker_host, 0, 256);
  // the relays' stream: one that, busy beside the best-effort stream, does not hold up the
  // high-priority stream
  c->side[c->n_side++] = c->be;
  if ((e = make_side_stream(c, &c->ctl)) != hipSuccess) {
    g_last_hip = (int)e;
    for (int i = 0; i < c->n_shunned; ++i) (void)hipStreamDestroy(c->shunned[i]);
    (void)hipFree(c->dev_pool);
    (void)hipFree(c->copy_pool);
    (void)hipHostFree(c->host_pool);
    (void)hipHostFree(c->marker_host);
    delete c;
    return TALLY_ERR_HIP;
  }
  c->be_delays_hi = delays_hi_stream(c, c->be, nullptr, 0);
  c->cur_be = c->be;
  c->cur_ctl = c->ctl;
  c->num_cus = (uint32_t)prop.multiProcessorCount;
  c->lds_per_cu = (uint32_t)prop.maxSharedMemoryPerMultiProcessor;
  c->yield_ticks = 100000;  // 1 ms
  c->yield_every = 4;
  c->device = dev;
  for (int k = 0; k < TALLY_K_COUNT; ++k) {
    if (kOps[k].init && (e = kOps[k].init()) != hipSuccess) {
      g_last_hip = (int)e;
      tally_destroy(c);
      return TALLY_ERR_HIP;
    }
    for (int f = 0; f < 2; ++f) {
      uint32_t *ft = c->foot[k][f];
      ft[0] = 0; ft[1] = 4; ft[2] = 128;
      auto fn = f == 0 ? kOps[k].footprint : kOps[k].footprint_native;
      if (fn && (e = fn(&ft[0], &ft[1], &ft[2])) != hipSuccess) {
        g_last_hip = (int)e;
        tally_destroy(c);
        return TALLY_ERR_HIP;
      }
    }
    int per_cu = 0;
    c->max_workers[k] = 0;
    if (kOps[k].occupancy) {
      if (kOps[k].occupancy(&per_cu) != TALLY_OK || per_cu < 1) {
        tally_destroy(c);
        return TALLY_ERR_HIP;
      }
      c->max_workers[k] = (uint32_t)per_cu * c->num_cus;
    }
  }
  if ((e = attn_decode_init()) != hipSuccess) {
    g_last_hip = (int)e;
    tally_destroy(c);
    return TALLY_ERR_HIP;
  }
  *out = c;
  return TALLY_OK;
}

int tally_destroy(tally_ctx *ctx) {
  if (!ctx) return TALLY_ERR_INVALID_ARG;
  if (ctx->live_jobs != 0) return TALLY_ERR_BAD_STATE;
  (void)hipStreamSynchronize(ctx->hi);
  (void)hipStreamSynchronize(ctx->be);
  (void)hipStreamSynchronize(ctx->ctl);
  (void)hipStreamDestroy(ctx->ctl);
  for (int i = 0; i < ctx->n_shunned; ++i) (void)hipStreamDestroy(ctx->shunned[i]);
  for (int i = 0; i < kMaxBeClients; ++i) {
    if (ctx->client_be[i]) { (void)hipStreamSynchronize(ctx->client_be[i]); (void)hipStreamDestroy(ctx->client_be[i]); }
    if (ctx->client_ctl[i]) { (void)hipStreamSynchronize(ctx->client_ctl[i]); (void)hipStreamDestroy(ctx->client_ctl[i]); }
  }
  (void)hipFree(ctx->dev_pool);
  (void)hipFree(ctx->copy_pool);
  (void)hipHostFree(ctx->host_pool);
  (void)hipHostFree(ctx->marker_host);
  delete ctx;
  return TALLY_OK;
}

int tally_logical_grid(uint32_t kernel_id, const void *args, size_t args_size, tally_dim3 *grid,
                       tally_dim3 *block) {
  if (kernel_id >= TALLY_K_COUNT || !args || !grid || !block) return TALLY_ERR_INVALID_ARG;
  if (args_size != kOps[kernel_id].args_size) return TALLY_ERR_INVALID_ARG;
  tally_dim3 g, b;
  int rc = kOps[kernel_id].grid(args, &g, &b);
  if (rc) return rc;
  *grid = g;
  *block = b;
  return TALLY_OK;
}

size_t tally_attn_decode_scratch_bytes(uint32_t heads) { return attn_decode_scratch_bytes(heads); }

int tally_launch_native(tally_ctx *ctx, const tally_kernel_desc *desc, int on_hi_stream) {
  if (!ctx) return TALLY_ERR_INVALID_ARG;
  const KernelOps *ops;
  tally_dim3 g;
  int rc = check_desc(desc, &ops, &g);
  if (rc) return rc;
  HIPCHK(ops->native(on_hi_stream ? ctx->hi : ctx->be, desc->args, g, on_hi_stream ? 1u : 0u));
  return TALLY_OK;
}

int tally_launch_attn_decode_static(tally_ctx *ctx, const tally_attn_decode_args *args,
                                    int on_hi_stream) {
  if (!ctx || !args) return TALLY_ERR_INVALID_ARG;
  if (args->heads > kStaticAttnMaxHeads) return TALLY_ERR_INVALID_ARG;
  tally_attn_decode_args a = *args;
  a.scratch = ctx->static_attn_scratch;  // the address obtained at tally_create, never the symbol
  tally_dim3 g, b;
  int rc = grid_attn(&a, &g, &b);
  if (rc) return rc;
  int dev = -1;
  HIPCHK(hipGetDevice(&dev));
  if (dev != ctx->device) return TALLY_ERR_BAD_STATE;  // each GPU has its own copy of the array
  HIPCHK(launch_attn_decode(on_hi_stream ? ctx->hi : ctx->be, &a, g, on_hi_stream ? 1u : 0u));
  return TALLY_OK;
}

int tally_launch_sliced(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t slice_blocks,
                        uint32_t max_in_flight, int coverage, tally_job **out) {
  if (!ctx || !out || slice_blocks == 0 || max_in_flight == 0) return TALLY_ERR_INVALID_ARG;
  tally_job *j;
  int rc = new_job(ctx, desc, KIND_SLICED, coverage, &j);
  if (rc) return rc;
  j->slice_blocks = slice_blocks;
  j->max_in_flight = max_in_flight;
  j->state = TALLY_JOB_RUNNING;
  rc = sliced_issue(j);
  if (rc) { tally_job_free(j); return rc; }
  *out = j;
  return TALLY_OK;
}

int tally_launch_ptb_until(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t num_workers,
                           uint32_t chunk, uint64_t stop_at, int coverage, tally_job **out) {
  if (!ctx || !out || !desc || num_workers == 0 || chunk == 0) return TALLY_ERR_INVALID_ARG;
  if (desc->kernel_id >= TALLY_K_COUNT || chunk > (1u << 16)) return TALLY_ERR_INVALID_ARG;
  // every worker resident at once (an unsupported kernel is reported by new_job below)
  if (kOps[desc->kernel_id].transformable && num_workers > ctx->max_workers[desc->kernel_id])
    return TALLY_ERR_INVALID_ARG;
  tally_job *j;
  int rc = new_job(ctx, desc, KIND_PTB, coverage, &j);
  if (rc) return rc;
  j->workers = num_workers;
  j->chunk = chunk;
  rc = ptb_launch_segment(j, stop_at > j->total ? j->total : (uint32_t)stop_at);
  if (rc) { tally_job_free(j); return rc; }
  *out = j;
  return TALLY_OK;
}

int tally_launch_ptb(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t num_workers,
                     uint32_t chunk, int coverage, tally_job **out) {
  return tally_launch_ptb_until(ctx, desc, num_workers, chunk, ~0ull, coverage, out);
}

int tally_mfma_ceiling_tflops(tally_ctx *ctx, uint32_t reps, double *tflops) {
  if (!ctx || !tflops || reps == 0 || reps > 1000) return TALLY_ERR_INVALID_ARG;
  uint4 *ops = nullptr;
  float *sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  uint32_t bits[512];
  uint32_t s = 1;
  for (int i = 0; i < 512; ++i) {  // pairs of small bf16 values of either sign
    s = s * 1664525u + 1013904223u;
    bits[i] = (s & 0x807F807Fu) | 0x3C003C00u;
  }
  const uint32_t iters = 256;  // x 16 accumulators = 4096 MFMAs per wave
  hipError_t e;
  int rc = TALLY_OK;
  float best_ms = 1e30f;
  if ((e = hipMalloc((void **)&ops, sizeof(bits))) != hipSuccess ||
      (e = hipMalloc((void **)&sink, (size_t)ctx->num_cus * 256 * sizeof(float))) != hipSuccess ||
      (e = hipMemcpy(ops, bits, sizeof(bits), hipMemcpyHostToDevice)) != hipSuccess ||
      (e = hipEventCreate(&e0)) != hipSuccess || (e = hipEventCreate(&e1)) != hipSuccess) {
    g_last_hip = (int)e;
    rc = TALLY_ERR_HIP;
  }
  for (uint32_t r = 0; rc == TALLY_OK && r < reps + 2; ++r) {  // two warm-up launches
    (void)hipEventRecord(e0, ctx->be);
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(ctx->num_cus), dim3(256), 0, ctx->be, ops, sink, iters);
    (void)hipEventRecord(e1, ctx->be);
    float ms = 0.f;
    if ((e = hipEventSynchronize(e1)) != hipSuccess || (e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) {
      g_last_hip = (int)e;
      rc = TALLY_ERR_HIP;
    } else if (r >= 2 && ms < best_ms) {
      best_ms = ms;
    }
  }
  if (rc == TALLY_OK)
    *tflops = (double)ctx->num_cus * 4 * 16 * iters * 32768.0 / (best_ms * 1e-3) / 1e12;
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (ops) (void)hipFree(ops);
  if (sink) (void)hipFree(sink);
  return rc;
}

int tally_kernel_footprint(tally_ctx *ctx, uint32_t kernel_id, int form, uint32_t *lds_bytes,
                           uint32_t *waves, uint32_t *regs_per_lane) {
  if (!ctx || kernel_id >= TALLY_K_COUNT || form < 0 || form > 1 || !lds_bytes || !waves || !regs_per_lane)
    return TALLY_ERR_INVALID_ARG;
  if (form == 0 && !kOps[kernel_id].transformable) return TALLY_ERR_UNSUPPORTED;
  *lds_bytes = ctx->foot[kernel_id][form][0];
  *waves = ctx->foot[kernel_id][form][1];
  *regs_per_lane = ctx->foot[kernel_id][form][2];
  return TALLY_OK;
}

int tally_max_workers(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t *max_workers) {
  if (!ctx || !desc || !max_workers || desc->kernel_id >= TALLY_K_COUNT) return TALLY_ERR_INVALID_ARG;
  if (!kOps[desc->kernel_id].transformable) return TALLY_ERR_UNSUPPORTED;
  *max_workers = ctx->max_workers[desc->kernel_id];
  return TALLY_OK;
}

namespace {
int preempt_impl(tally_job *job, bool pause) {
  if (!job) return TALLY_ERR_INVALID_ARG;
  if (job->state.load() != TALLY_JOB_RUNNING) return TALLY_OK;
  if (job->t_preempt.load() == 0.0) job->t_preempt = now_us();
  if (job->kind == KIND_PTB) {
    const uint32_t word = pause ? job->epoch : (job->epoch | kNoPauseBit);
    job->request_word = word;
    __atomic_store_n(job->h_flag(), word, __ATOMIC_RELEASE);
  } else if (job->kind == KIND_SLICED) {
    job->stop_issuing = true;
  }
  return TALLY_OK;
}
}  // namespace

int tally_preempt(tally_job *job) { return preempt_impl(job, false); }
int tally_preempt_pausing(tally_job *job) { return preempt_impl(job, true); }

int tally_resume_until(tally_job *job, uint64_t stop_at) {
  if (!job) return TALLY_ERR_INVALID_ARG;
  refresh(job);
  int st = job->state.load();
  if (st == TALLY_JOB_COMPLETE) return TALLY_OK;
  if (st != TALLY_JOB_STOPPED) return TALLY_ERR_BAD_STATE;
  if (job->kind == KIND_PTB) {
    if (stop_at < job->progress.load()) return TALLY_ERR_INVALID_ARG;
    return ptb_launch_segment(job, stop_at > job->total ? job->total : (uint32_t)stop_at);
  }
  job->stop_issuing = false;
  job->segment += 1;
  job->t_preempt = 0.0;
  job->state = TALLY_JOB_RUNNING;
  return sliced_issue(job);
}

int tally_resume(tally_job *job) { return tally_resume_until(job, ~0ull); }

int tally_end_pause(tally_job *job) {
  if (!job) return TALLY_ERR_INVALID_ARG;
  // Workers pausing inside a block go on and finish it.  The request itself is in the task
  // counter and cannot be taken back: every worker still leaves at its next block boundary
  // and the job then needs a resume like any preempted one.  The time of the request is
  // kept: the drain that follows is the preemption's.
  const uint32_t w = job->request_word.load();
  if (job->kind == KIND_PTB && w != 0 && !(w & kNoPauseBit) && job->state.load() == TALLY_JOB_RUNNING) {
    job->request_word = w | kNoPauseBit;
    __atomic_store_n(job->h_flag(), w | kNoPauseBit, __ATOMIC_RELEASE);
  }
  return TALLY_OK;
}

int tally_progress(tally_job *job, uint64_t *done_blocks, uint64_t *total_blocks, int *state) {
  if (!job) return TALLY_ERR_INVALID_ARG;
  // read-only view: safe from any thread (the owning thread advances the state)
  uint64_t p = job->progress.load();
  int st = job->state.load();
  if (st == TALLY_JOB_RUNNING && job->kind == KIND_PTB) {
    uint32_t live = __atomic_load_n(job->h_live(), __ATOMIC_RELAXED);
    if (live > p) p = live;
  }
  if (done_blocks) *done_blocks = p;
  if (total_blocks) *total_blocks = job->total;
  if (state) *state = st;
  return TALLY_OK;
}

int tally_pump(tally_job *job) {
  if (!job) return TALLY_ERR_INVALID_ARG;
  refresh(job);
  if (job->state.load() == TALLY_JOB_RUNNING && job->kind == KIND_SLICED) return sliced_issue(job);
  return TALLY_OK;
}

int tally_wait(tally_job *job, int *state) {
  if (!job) return TALLY_ERR_INVALID_ARG;
  for (uint32_t spins = 1;; ++spins) {
    int rc = tally_pump(job);
    if (rc) return rc;
    int st = job->state.load();
    if (job->failed) return TALLY_ERR_BAD_STATE;
    if (st == TALLY_JOB_STOPPED || st == TALLY_JOB_COMPLETE) break;
    // a kernel that failed after enqueue would leave the status word unwritten for ever
    if ((spins & 0xFFFFu) == 0) {
      hipError_t q = hipStreamQuery(job->be);
      if (q != hipSuccess && q != hipErrorNotReady) { g_last_hip = (int)q; return TALLY_ERR_HIP; }
    }
  }
  HIPCHK(hipStreamSynchronize(job->be));
  if (state) *state = job->state.load();
  return TALLY_OK;
}

int tally_job_free(tally_job *job) {
  if (!job) return TALLY_ERR_INVALID_ARG;
  tally_ctx *ctx = job->ctx;
  if (job->state.load() == TALLY_JOB_RUNNING) {
    job->stop_issuing = true;
    (void)hipStreamSynchronize(job->be);
  }
  if (job->cover) {
    (void)hipStreamSynchronize(job->be);
    (void)hipFree(job->cover);
  }
  if (job->kind == KIND_PTB) {
    // the slot's counter may not be handed to another job before this job's last relay has
    // ended (it could still fold a late request in) and has reported the counter's value
    refresh(job);
    (void)settle_relay(job);
  }
  ctx->slot_used[job->slot] = false;
  ctx->live_jobs--;
  delete job;
  return TALLY_OK;
}

int tally_coverage(tally_job *job, void *host_records, size_t bytes) {
  if (!job || !host_records || !job->cover) return TALLY_ERR_INVALID_ARG;
  if (bytes != sizeof(tally_cover_rec) * (size_t)job->total) return TALLY_ERR_INVALID_ARG;
  refresh(job);
  if (job->state.load() == TALLY_JOB_RUNNING) return TALLY_ERR_BAD_STATE;
  HIPCHK(hipStreamSynchronize(job->be));
  HIPCHK(hipMemcpy(host_records, job->cover, bytes, hipMemcpyDeviceToHost));
  return TALLY_OK;
}

int tally_marker(tally_ctx *ctx, int on_hi_stream, uint32_t value) {
  if (!ctx) return TALLY_ERR_INVALID_ARG;
  hipLaunchKernelGGL(marker_kernel, dim3(1), dim3(64), 0, on_hi_stream ? ctx->hi : ctx->be,
                     ctx->marker_dev + (on_hi_stream ? 0 : 32), value);
  HIPCHK(hipGetLastError());
  return TALLY_OK;
}

int tally_marker_read(tally_ctx *ctx, int on_hi_stream, uint32_t *value) {
  if (!ctx || !value) return TALLY_ERR_INVALID_ARG;
  *value = __atomic_load_n(ctx->marker_host + (on_hi_stream ? 0 : 32), __ATOMIC_ACQUIRE);
  return TALLY_OK;
}

int tally_last_preempt_latency_us(tally_job *job, double *us) {
  if (!job || !us) return TALLY_ERR_INVALID_ARG;
  *us = job->preempt_latency_us;
  return TALLY_OK;
}

int tally_set_yield_bound_us(tally_ctx *ctx, uint32_t us) {
  if (!ctx || us > 1000000u) return TALLY_ERR_INVALID_ARG;
  ctx->yield_ticks = us * 100u;
  return TALLY_OK;
}

int tally_set_yield_every(tally_ctx *ctx, uint32_t steps) {
  if (!ctx || steps == 0 || steps > 1024 || (steps & (steps - 1))) return TALLY_ERR_INVALID_ARG;
  ctx->yield_every = steps;
  return TALLY_OK;
}

int tally_last_hip_error(void) { return g_last_hip; }

const char *tally_strerror(int status) {
  switch (status) {
    case TALLY_OK: return "ok";
    case TALLY_ERR_INVALID_ARG: return "invalid argument";
    case TALLY_ERR_BAD_STATE: return "operation not valid in the job's current state";
    case TALLY_ERR_HIP: return "HIP call failed";
    case TALLY_ERR_NOMEM: return "out of memory or job slots";
    case TALLY_ERR_UNSUPPORTED: return "kernel cannot be sliced or preempted";
    default: return "unknown status";
  }
}

int tally_device_info(uint32_t *num_cus, uint32_t *lds_bytes_per_cu, uint32_t *wave_size) {
  int dev = 0;
  hipDeviceProp_t prop;
  HIPCHK(hipGetDevice(&dev));
  HIPCHK(hipGetDeviceProperties(&prop, dev));
  if (num_cus) *num_cus = (uint32_t)prop.multiProcessorCount;
  if (lds_bytes_per_cu) *lds_bytes_per_cu = (uint32_t)prop.maxSharedMemoryPerMultiProcessor;
  if (wave_size) *wave_size = (uint32_t)prop.warpSize;
  return TALLY_OK;
}

int tally_stream_report(tally_ctx *ctx, int *be_delays_hi, uint32_t *set_aside) {
  if (!ctx) return TALLY_ERR_INVALID_ARG;
  if (be_delays_hi) *be_delays_hi = (ctx->be_delays_hi ? 1 : 0) | (ctx->side_crowded ? 2 : 0);
  if (set_aside) *set_aside = (uint32_t)ctx->n_shunned;
  return TALLY_OK;
}

// ------------------------------------------------------------------ configuration choice
double tally_ptb_turnaround_ms(double kernel_latency_ms, uint32_t worker_blocks, uint32_t chunk,
                               uint64_t total_blocks) {
  if (total_blocks == 0) return 0.0;
  return kernel_latency_ms * (double)worker_blocks * (double)(chunk ? chunk : 1) /
         (double)total_blocks;
}

int tally_select_config(const tally_config *c, uint32_t n, double threshold_ms) {
  if (!c || n == 0) return TALLY_ERR_INVALID_ARG;
  // order of preference among equals: persistent workers first, then fewer workers,
  // then larger slices
  auto better_tie = [&](const tally_config &x, const tally_config &y) {
    if (x.kind != y.kind) return x.kind < y.kind;
    return x.kind == 0 ? x.param < y.param : x.param > y.param;
  };
  int best = -1;
  for (uint32_t i = 0; i < n; ++i) {
    if (c[i].turnaround_ms > threshold_ms) continue;
    if (best < 0 || c[i].latency_ms < c[best].latency_ms ||
        (c[i].latency_ms == c[best].latency_ms && better_tie(c[i], c[best])))
      best = (int)i;
  }
  if (best >= 0) return best;
  best = 0;
  for (uint32_t i = 1; i < n; ++i)
    if (c[i].turnaround_ms < c[best].turnaround_ms ||
        (c[i].turnaround_ms == c[best].turnaround_ms && better_tie(c[i], c[best])))
      best = (int)i;
  return best;
}

}  // extern "C"

namespace {

ProfileKey profile_key(const tally_kernel_desc *d) {
  return std::make_tuple(d->kernel_id, d->grid.x, d->grid.y, d->grid.z, d->block.x);
}

// Turnaround estimate of one measured candidate (Section 4.2).
void fill_turnaround(tally_ctx *ctx, const KernelOps *ops, const void *args, uint64_t total,
                     tally_config *c) {
  if (c->kind == 0) {
    c->turnaround_ms = (float)tally_ptb_turnaround_ms(c->latency_ms, c->param, c->chunk ? c->chunk : 1, total);
    // a body that pauses inside its blocks hands the execution units over after a share
    // of ONE block, whatever the chunk: Eq. 1 with chunk 1, times that share
    const double share = ctx->yield_ticks ? ops->pause_fraction(args, ctx->yield_every) : 1.0;
    if (share < 1.0)
      c->turnaround_ms = (float)(tally_ptb_turnaround_ms(c->latency_ms, c->param, 1, total) * share);
  } else {
    // one slice's time, times the number of slices that may be enqueued at once
    uint64_t slices = (total + c->param - 1) / c->param;
    uint64_t inflight = c->chunk ? c->chunk : 1;
    if (inflight > slices) inflight = slices;
    c->turnaround_ms = (float)(c->latency_ms / (double)slices * (double)inflight);
  }
}

// The candidate set of Section 4.2: persistent-worker counts that are multiples of the
// compute-unit count and fit (every worker resident), each with 1, 4 and 16 task indices per
// fetch where the grid has that many blocks per worker; slices of 1/2 ... 1/256 of the grid.
uint32_t candidate_configs(tally_ctx *ctx, uint32_t kernel_id, uint64_t total, tally_config *out,
                           uint32_t cap) {
  uint32_t n = 0;
  auto push = [&](uint32_t kind, uint32_t param, uint32_t chunk) {
    for (uint32_t i = 0; i < n; ++i)
      if (out[i].kind == kind && out[i].param == param && out[i].chunk == chunk) return;
    if (n < cap) out[n++] = tally_config{kind, param, chunk, 0.f, 0.f};
  };
  const uint32_t maxw = ctx->max_workers[kernel_id];
  for (uint32_t w = ctx->num_cus; w <= maxw; w += ctx->num_cus) {
    const uint32_t workers = (uint64_t)w < total ? w : (uint32_t)total;
    static const uint32_t chunks[3] = {1, 4, 16};
    for (uint32_t ch : chunks)
      if (ch == 1 || (uint64_t)workers * ch <= total) push(0, workers, ch);
    if ((uint64_t)w >= total) break;
  }
  // the whole grid as one slice first: a kernel shorter than the threshold complies as it is
  for (uint32_t sh = 0; sh <= 8; ++sh) {
    const uint64_t blocks = total >> sh;
    push(1, (uint32_t)(blocks ? blocks : 1), 1);
  }
  return n;
}

// Record one measurement; when the table is complete, choose.  Returns true when the
// configuration became fixed by this call.
bool profile_record(tally_ctx *ctx, ProfileEntry &e, uint32_t idx, double ms, uint32_t runs,
                    double threshold_ms, const KernelOps *ops, const void *args, uint64_t total) {
  e.sum_ms[idx] += ms;
  e.samples[idx] += 1;
  for (uint32_t i = 0; i < e.cands.size(); ++i)
    if (e.samples[i] < runs) return false;
  for (uint32_t i = 0; i < e.cands.size(); ++i) {
    e.cands[i].latency_ms = (float)(e.sum_ms[i] / e.samples[i]);
    fill_turnaround(ctx, ops, args, total, &e.cands[i]);
  }
  e.chosen = tally_select_config(e.cands.data(), (uint32_t)e.cands.size(), threshold_ms);
  e.threshold_ms = threshold_ms;
  return true;
}

}  // namespace

extern "C" {

int tally_candidate_configs(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *out,
                            uint32_t cap, uint32_t *n) {
  if (!ctx || !desc || !out || !n || cap == 0) return TALLY_ERR_INVALID_ARG;
  const KernelOps *ops;
  tally_dim3 g;
  int rc = check_desc(desc, &ops, &g);
  if (rc) return rc;
  if (!ops->transformable) return TALLY_ERR_UNSUPPORTED;
  *n = candidate_configs(ctx, desc->kernel_id, (uint64_t)g.x * g.y * g.z, out, cap);
  return TALLY_OK;
}

int tally_profile(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *cands, uint32_t n,
                  uint32_t runs, double threshold_ms, uint32_t *chosen) {
  if (!ctx || !desc || !cands || n == 0 || runs == 0) return TALLY_ERR_INVALID_ARG;
  const KernelOps *ops;
  tally_dim3 g;
  int rc = check_desc(desc, &ops, &g);
  if (rc) return rc;
  const uint64_t total = (uint64_t)g.x * g.y * g.z;
  ProfileEntry e;
  e.cands.assign(cands, cands + n);
  e.sum_ms.assign(n, 0.0);
  e.samples.assign(n, 0);
  for (uint32_t i = 0; i < n; ++i) {
    if (cands[i].kind > 1 || cands[i].param == 0) return TALLY_ERR_INVALID_ARG;
    for (uint32_t r = 0; r <= runs; ++r) {  // run 0 is the warm-up
      tally_be_item it = {desc, cands[i]};
      tally_job *j;
      HIPCHK(hipStreamSynchronize(ctx->be));
      double t0 = now_us();
      rc = launch_be_item(ctx, &it, &j);
      if (rc) return rc;
      int st;
      rc = tally_wait(j, &st);
      double t1 = now_us();
      tally_job_free(j);
      if (rc) return rc;
      if (r > 0) profile_record(ctx, e, i, (t1 - t0) / 1000.0, runs, threshold_ms, ops, desc->args, total);
    }
  }
  if (e.chosen < 0) return e.chosen;
  for (uint32_t i = 0; i < n; ++i) cands[i] = e.cands[i];
  if (chosen) *chosen = (uint32_t)e.chosen;
  std::lock_guard<std::mutex> lk(ctx->profile_mu);
  ctx->profiles[profile_key(desc)] = e;
  return TALLY_OK;
}

int tally_lookup_config(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *out) {
  if (!ctx || !desc || !out) return TALLY_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(ctx->profile_mu);
  auto it = ctx->profiles.find(profile_key(desc));
  if (it == ctx->profiles.end() || it->second.chosen < 0) return TALLY_ERR_BAD_STATE;
  *out = it->second.cands[it->second.chosen];
  return TALLY_OK;
}

int tally_profile_table(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *out, uint32_t cap,
                        uint32_t *n, uint32_t *samples, int *chosen) {
  if (!ctx || !desc || !n) return TALLY_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(ctx->profile_mu);
  auto it = ctx->profiles.find(profile_key(desc));
  if (it == ctx->profiles.end()) { *n = 0; if (chosen) *chosen = -1; return TALLY_OK; }
  const ProfileEntry &e = it->second;
  *n = (uint32_t)e.cands.size();
  for (uint32_t i = 0; i < *n && i < cap; ++i) {
    if (out) {
      out[i] = e.cands[i];
      if (e.samples[i]) out[i].latency_ms = (float)(e.sum_ms[i] / e.samples[i]);
    }
    if (samples) samples[i] = e.samples[i];
  }
  if (chosen) *chosen = e.chosen;
  return TALLY_OK;
}

int tally_profile_reset(tally_ctx *ctx) {
  if (!ctx) return TALLY_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(ctx->profile_mu);
  ctx->profiles.clear();
  return TALLY_OK;
}

}  // extern "C"

namespace {

int launch_be_item(tally_ctx *ctx, const tally_be_item *it, tally_job **out) {
  const tally_config &c = it->config;
  if (c.kind == 0) return tally_launch_ptb(ctx, it->kernel, c.param, c.chunk ? c.chunk : 1, 0, out);
  if (c.kind == 1) return tally_launch_sliced(ctx, it->kernel, c.param, c.chunk ? c.chunk : 1, 0, out);
  if (c.kind != 2) return TALLY_ERR_INVALID_ARG;
  tally_job *j;
  int rc = new_job(ctx, it->kernel, KIND_NATIVE, 0, &j);
  if (rc) return rc;
  j->state = TALLY_JOB_RUNNING;
  hipError_t e = j->ops->native(j->be, j->args, j->grid, 0u);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(marker_kernel, dim3(1), dim3(64), 0, j->be,
                       (uint32_t *)(j->h_base_dev() + 128), 1u);
    e = hipGetLastError();
  }
  if (e != hipSuccess) {
    g_last_hip = (int)e;
    tally_job_free(j);
    return TALLY_ERR_HIP;
  }
  *out = j;
  return TALLY_OK;
}

}  // namespace

// --------------------------------------------------------------- priority scheduling loop
// The loop of Figure 4, built on the public calls above (launch, preempt, resume, pump,
// progress), split over two host threads, one per client class, because a launch call cannot
// be interrupted: a single thread that is inside the best-effort client's launch when a
// high-priority kernel arrives delays it by that call.
//   high-priority client (the caller's thread, tally_sched_submit_hi / tally_sched_poll):
//     on arrival, preempt the running best-effort kernels, launch the request's kernels in
//     their original form, then watch for the completion marker.  While a request is in
//     flight `hi_active` is set.
//   best-effort clients (the scheduler's own thread): fetch the next kernel of each client,
//     look its configuration up or profile the next unmeasured candidate with this very
//     invocation, launch / resume / issue the next slice only while `hi_active` is clear;
//     account for completed kernels and preemption latencies.  The thread sleeps while no
//     client has work.
namespace {

constexpr uint32_t kCfgAuto = 3;   // tally_config.kind: let the profiler choose
constexpr uint32_t kPreemptRing = 4096;

struct BeWork {
  tally_kernel_desc desc;
  alignas(16) unsigned char args[kMaxArgs];
  tally_config config;     // kind kCfgAuto: profile-guided
  bool loop;               // goes to the back of its client's queue when it completes
  bool last_of_step;       // completing it ends one step of a looping client
};

// One best-effort client: its own queue of kernels, its own stream pair, one kernel in
// flight at a time (Figure 4 visits every best-effort client on every pass).
struct BeClient {
  std::deque<BeWork> queue;      // guarded by tally_sched::mu
  hipStream_t be = nullptr, ctl = nullptr;
  // `job` and the fields below it are written by the best-effort thread under `lock` and
  // read by the high-priority client under `lock`
  std::atomic_flag lock = ATOMIC_FLAG_INIT;
  tally_job *job = nullptr;
  BeWork cur;                    // the kernel in flight (or stopped)
  bool has_cur = false;
  int profiling = -1;            // candidate index this invocation measures, or -1
  double t_launch = 0.0;
  bool preempt_seen = false;     // a preemption request was raised against the current segment
  uint32_t dl = 0, dw = 0, dr = 0;   // per-compute-unit demand of its resident workgroups
  uint64_t ticket = 0;           // place in the queue of clients waiting for room (0: not waiting)
  std::atomic<uint64_t> kernels_done{0}, steps_done{0};
};

struct SpinGuard {
  std::atomic_flag &f;
  explicit SpinGuard(std::atomic_flag &fl) : f(fl) { while (f.test_and_set(std::memory_order_acquire)) {} }
  ~SpinGuard() { f.clear(std::memory_order_release); }
};

}  // namespace

struct tally_sched {
  tally_ctx *ctx;
  tally_sched_opts opts;
  double threshold_ms;
  uint32_t profile_runs;
  uint32_t n_clients;
  BeClient clients[kMaxBeClients];
  std::mutex mu;                      // queues, wake-ups
  std::condition_variable cv;
  std::thread be_thread;
  std::atomic<bool> hi_active{false}, stop{false}, be_enabled{true};
  std::atomic<double> t_preempt{0.0};
  std::atomic<int> rc{TALLY_OK};
  // the high-priority request in flight: largest demand of one of its workgroups
  uint32_t hl = 0, hw = 0, hr = 0;
  bool hi_inflight = false;
  uint32_t hi_seq = 0;
  uint64_t hi_done = 0;
  // statistics
  std::atomic<uint64_t> n_preempts{0}, profile_samples{0}, configs_fixed{0};
  std::mutex pre_mu;
  std::vector<double> pre_ring;
  uint64_t next_ticket = 0;
};

namespace {

// Per-compute-unit demand of the workgroups a best-effort kernel puts on the GPU at once
// (all its workers; one slice; the whole grid for a native launch), spread evenly.
int item_demand(tally_ctx *ctx, const tally_kernel_desc *desc, const tally_config &cfg, uint32_t *lds,
                uint32_t *waves, uint32_t *regs) {
  const KernelOps *ops;
  tally_dim3 g;
  int rc = check_desc(desc, &ops, &g);
  if (rc) return rc;
  const uint32_t *ft = ctx->foot[desc->kernel_id][cfg.kind == 0 ? 0 : 1];
  const uint32_t l = ft[0], w = ft[1], r = ft[2];
  const uint64_t total = (uint64_t)g.x * g.y * g.z;
  uint64_t groups = cfg.kind == 2 ? total : cfg.param;
  if (groups > total) groups = total;
  const uint64_t per_cu = (groups + ctx->num_cus - 1) / ctx->num_cus;
  const uint64_t cap = 64;  // beyond any compute unit's capacity: keeps the products small
  const uint32_t n = (uint32_t)(per_cu < cap ? per_cu : cap);
  *lds = n * l;
  *waves = n * w;
  *regs = n * ((w + 3) / 4) * r;  // per SIMD: a workgroup's waves go round the four SIMDs
  return TALLY_OK;
}

// lookup_launch_config() / launch_and_profile() of Figure 4 for one fetched kernel: the
// configuration to launch this invocation with, and which candidate (if any) the
// invocation measures.  One unmeasured candidate is profiled per real invocation; once
// every candidate has its samples the choice is made and kept (Section 4.2).
int choose_config(tally_sched *s, const BeWork &w, tally_config *cfg, int *profiling) {
  *profiling = -1;
  if (w.config.kind != kCfgAuto) { *cfg = w.config; return TALLY_OK; }
  tally_ctx *ctx = s->ctx;
  std::lock_guard<std::mutex> lk(ctx->profile_mu);
  ProfileEntry &e = ctx->profiles[profile_key(&w.desc)];
  if (e.cands.empty()) {
    tally_config tmp[64];
    const uint64_t total = (uint64_t)w.desc.grid.x * w.desc.grid.y * w.desc.grid.z;
    uint32_t n = candidate_configs(ctx, w.desc.kernel_id, total, tmp, 64);
    if (n == 0) return TALLY_ERR_UNSUPPORTED;
    e.cands.assign(tmp, tmp + n);
    e.sum_ms.assign(n, 0.0);
    e.samples.assign(n, 0);
  }
  if (e.chosen >= 0) {
    if (e.threshold_ms != s->threshold_ms) {   // the threshold moved: choose again from the table
      e.chosen = tally_select_config(e.cands.data(), (uint32_t)e.cands.size(), s->threshold_ms);
      e.threshold_ms = s->threshold_ms;
    }
    *cfg = e.cands[e.chosen];
    return TALLY_OK;
  }
  for (uint32_t i = 0; i < e.cands.size(); ++i)
    if (e.samples[i] < s->profile_runs) {
      *cfg = e.cands[i];
      *profiling = (int)i;
      return TALLY_OK;
    }
  return TALLY_ERR_BAD_STATE;  // unreachable: a full table has a choice
}

void be_thread_main(tally_sched *s) {
  tally_ctx *ctx = s->ctx;
  int rc = TALLY_OK;
  if (hipSetDevice(ctx->device) != hipSuccess) { s->rc = TALLY_ERR_HIP; return; }
  // A kernel is put on the GPU only if all the workgroups it brings fit beside the
  // best-effort workgroups already resident: a dispatch that waits for resources blocks
  // its hardware pipe for every queue mapped to that pipe, the high-priority queue
  // possibly among them (two 128 KB-LDS GEMMs launched together held high-priority
  // kernels back for milliseconds).  Clients that have to wait are served first come,
  // first served.  A client with the GPU to itself is always admitted.
  auto admit = [&](uint32_t c, uint32_t l, uint32_t w, uint32_t r) -> bool {
    BeClient &cl = s->clients[c];
    if (cl.ticket == 0) cl.ticket = ++s->next_ticket;
    uint32_t lds = 0, waves = 0, regs = 0, others = 0;
    for (uint32_t o = 0; o < s->n_clients; ++o) {
      if (o == c) continue;
      const BeClient &oc = s->clients[o];
      if (oc.ticket != 0 && oc.ticket < cl.ticket) return false;
      if (oc.dw) others++;
      lds += oc.dl;
      waves += oc.dw;
      regs += oc.dr;
    }
    // (one wave slot and 32 registers are kept back for the newcomer's relay)
    if (others && (lds + l > ctx->lds_per_cu || waves + w > 31u || regs + r > 480u)) return false;
    SpinGuard g(cl.lock);
    cl.dl = l; cl.dw = w; cl.dr = r;
    cl.ticket = 0;
    return true;
  };
  auto vacate = [&](BeClient &cl) { SpinGuard g(cl.lock); cl.dl = cl.dw = cl.dr = 0; };
  auto set_job = [&](BeClient &cl, tally_job *j) { SpinGuard g(cl.lock); cl.job = j; };
  auto note_preempt = [&](double us) {
    s->n_preempts++;
    std::lock_guard<std::mutex> lk(s->pre_mu);
    if (s->pre_ring.size() < kPreemptRing) s->pre_ring.push_back(us);
  };
  auto finish = [&](BeClient &cl, bool completed) {
    tally_job *j = cl.job;
    if (completed && cl.profiling >= 0 && j->segments <= 1 && j->segment == 0 && !cl.preempt_seen) {
      // this invocation was the measurement of one candidate (and was not disturbed)
      const KernelOps *ops = j->ops;
      std::lock_guard<std::mutex> lk(ctx->profile_mu);
      ProfileEntry &e = ctx->profiles[profile_key(&cl.cur.desc)];
      if (e.chosen < 0 && (size_t)cl.profiling < e.cands.size()) {
        s->profile_samples++;
        if (profile_record(ctx, e, (uint32_t)cl.profiling, (now_us() - cl.t_launch) / 1000.0,
                           s->profile_runs, s->threshold_ms, ops, cl.cur.args, j->total))
          s->configs_fixed++;
      }
    }
    set_job(cl, nullptr);
    tally_job_free(j);
    vacate(cl);
    cl.preempt_seen = false;
    cl.profiling = -1;
    if (completed) {
      cl.kernels_done++;
      if (cl.cur.last_of_step) cl.steps_done++;
      if (cl.cur.loop) {
        std::lock_guard<std::mutex> lk(s->mu);
        cl.queue.push_back(cl.cur);
      }
    }
    cl.has_cur = false;
  };

  while (rc == TALLY_OK) {
    const bool stopping = s->stop.load();
    uint32_t busy = 0;
    for (uint32_t c = 0; c < s->n_clients && rc == TALLY_OK; ++c) {
      BeClient &cl = s->clients[c];
      const bool closing = stopping || !s->be_enabled.load();
      const bool hold = s->opts.policy != 2 && s->hi_active.load();
      if (cl.job) {
        tally_job *be = cl.job;
        busy++;
        if (hold && !cl.preempt_seen && be->state.load() == TALLY_JOB_RUNNING) {
          // the high-priority client raised the request (persistent workers); for the other
          // kinds "preempt" means that nothing further is issued until the request is done
          cl.preempt_seen = true;
          if (be->t_preempt.load() == 0.0) be->t_preempt = s->t_preempt.load();
          if (be->kind == KIND_SLICED) be->stop_issuing = true;
        }
        rc = tally_pump(be);   // refresh; a sliced job also issues its next slice unless stopped
        if (rc) break;
        if (be->failed) { rc = TALLY_ERR_BAD_STATE; break; }
        const int st = be->state.load();
        if (st == TALLY_JOB_COMPLETE) {
          finish(cl, true);
        } else if (st == TALLY_JOB_STOPPED) {
          vacate(cl);
          if (cl.preempt_seen && be->preempt_latency_us >= 0.0) note_preempt(be->preempt_latency_us);
          cl.preempt_seen = false;
          if (stopping) {
            finish(cl, false);
          } else if (closing) {
            // best-effort work is switched off: the kernel stays stopped where it is
          } else if (!hold) {
            uint32_t l = 0, w = 0, r = 0;
            tally_config cfg{};
            cfg.kind = (uint32_t)be->kind;
            cfg.param = be->kind == KIND_PTB ? be->workers : be->slice_blocks;
            (void)item_demand(ctx, &cl.cur.desc, cfg, &l, &w, &r);
            if (admit(c, l, w, r)) {
              rc = tally_resume(be);   // kernel.resume()
              if (rc) break;
              // a request that arrived while the resume was being made saw a stopped job
              if (s->opts.policy == 0 && s->hi_active.load() && be->kind == KIND_PTB) {
                be->t_preempt = s->t_preempt.load();
                (void)tally_preempt(be);
                cl.preempt_seen = true;
              }
            }
          }
        } else if (closing) {
          // shutting down: drain at block boundaries, without pausing
          if (be->kind == KIND_SLICED) be->stop_issuing = true;
          else if (be->kind == KIND_PTB) (void)tally_preempt(be);
        }
      }
      if (!cl.job && !stopping && s->be_enabled.load()) {
        if (!cl.has_cur) {
          std::lock_guard<std::mutex> lk(s->mu);
          if (!cl.queue.empty()) {             // client.fetch_next_kernel()
            cl.cur = cl.queue.front();
            cl.queue.pop_front();
            cl.cur.desc.args = cl.cur.args;
            cl.has_cur = true;
          }
        }
        if (cl.has_cur) busy++;
        if (cl.has_cur && !hold) {
          tally_config cfg;
          int prof = -1;
          rc = choose_config(s, cl.cur, &cfg, &prof);
          if (rc) break;
          uint32_t l = 0, w = 0, r = 0;
          (void)item_demand(ctx, &cl.cur.desc, cfg, &l, &w, &r);
          if (admit(c, l, w, r)) {
            ctx->cur_be = cl.be;
            ctx->cur_ctl = cl.ctl;
            tally_be_item it = {&cl.cur.desc, cfg};
            tally_job *j = nullptr;
            cl.t_launch = now_us();
            rc = launch_be_item(ctx, &it, &j);
            ctx->cur_be = ctx->be;
            ctx->cur_ctl = ctx->ctl;
            if (rc) break;
            cl.profiling = prof;
            set_job(cl, j);
            // a request that arrived while this launch was being made found no job to
            // preempt: raise it against the new segment here
            if (s->opts.policy == 0 && s->hi_active.load() && j->kind == KIND_PTB) {
              j->t_preempt = s->t_preempt.load();
              (void)tally_preempt(j);
              cl.preempt_seen = true;
            }
          }
        }
      }
    }
    if (stopping && busy == 0) break;
    // kernels in flight: the loop watches their status words; tell the core it is a spin
    // wait (a sibling hardware thread, the high-priority client's perhaps, gets the issue slots)
    if (busy != 0) __builtin_ia32_pause();
    if (busy == 0) {
      // nothing in flight and nothing queued: sleep until a kernel is submitted
      std::unique_lock<std::mutex> lk(s->mu);
      bool any = false;
      for (uint32_t c = 0; c < s->n_clients; ++c) any = any || !s->clients[c].queue.empty();
      if (!any && !s->stop.load())
        s->cv.wait_for(lk, std::chrono::milliseconds(50));
    }
  }
  for (uint32_t c = 0; c < s->n_clients; ++c) {
    BeClient &cl = s->clients[c];
    if (cl.job) {
      tally_job *j = cl.job;
      set_job(cl, nullptr);
      tally_job_free(j);
    }
  }
  if (rc) s->rc = rc;
}

}  // namespace

extern "C" {

int tally_sched_create(tally_ctx *ctx, const tally_sched_opts *opts, tally_sched **out) {
  if (!ctx || !opts || !out) return TALLY_ERR_INVALID_ARG;
  if (opts->policy > 2 || opts->n_be_clients > (uint32_t)kMaxBeClients) return TALLY_ERR_INVALID_ARG;
  if (opts->threshold_ms < 0.0) return TALLY_ERR_INVALID_ARG;
  const uint32_t n_clients = opts->n_be_clients;
  // Every client needs two hardware queues (kernels, relays) beside the null stream's and
  // the high-priority stream's.  HIP folds streams onto GPU_MAX_HW_QUEUES hardware queues
  // (4 unless the environment says otherwise), and streams that share one run in order:
  // a high-priority kernel behind a relay would wait for a whole best-effort kernel.
  if (n_clients >= 1) {
    const char *env = getenv("GPU_MAX_HW_QUEUES");
    const long have = env ? strtol(env, nullptr, 10) : 4;
    if (have < (long)(2 + 2 * n_clients)) return TALLY_ERR_UNSUPPORTED;
  }
  tally_sched *s = new (std::nothrow) tally_sched();
  if (!s) return TALLY_ERR_NOMEM;
  s->ctx = ctx;
  s->opts = *opts;
  s->threshold_ms = opts->threshold_ms > 0.0 ? opts->threshold_ms : 0.0316;
  s->profile_runs = opts->profile_runs ? opts->profile_runs : 10;
  s->n_clients = n_clients;
  for (uint32_t c = 0; c < n_clients; ++c) {
    if (c == 0) {
      s->clients[c].be = ctx->be;
      s->clients[c].ctl = ctx->ctl;
    } else {  // further clients get a stream pair of their own, made once per context
      hipError_t e = hipSuccess;
      if (!ctx->client_be[c]) e = make_side_stream(ctx, &ctx->client_be[c]);
      if (e == hipSuccess && !ctx->client_ctl[c]) e = make_side_stream(ctx, &ctx->client_ctl[c]);
      if (e != hipSuccess) { g_last_hip = (int)e; delete s; return TALLY_ERR_HIP; }
      s->clients[c].be = ctx->client_be[c];
      s->clients[c].ctl = ctx->client_ctl[c];
    }
  }
  hipError_t e = hipStreamSynchronize(ctx->hi);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->be);
  if (e != hipSuccess) { g_last_hip = (int)e; delete s; return TALLY_ERR_HIP; }
  (void)tally_marker_read(ctx, 1, &s->hi_seq);
  if (n_clients) s->be_thread = std::thread(be_thread_main, s);
  *out = s;
  return TALLY_OK;
}

int tally_sched_destroy(tally_sched *s) {
  if (!s) return TALLY_ERR_INVALID_ARG;
  s->stop = true;
  s->hi_active = false;
  s->cv.notify_all();
  if (s->be_thread.joinable()) s->be_thread.join();
  for (uint32_t c = 0; c < s->n_clients; ++c) (void)hipStreamSynchronize(s->clients[c].be);
  (void)hipStreamSynchronize(s->ctx->hi);
  (void)hipStreamSynchronize(s->ctx->be);
  int rc = s->rc.load();
  delete s;
  return rc;
}

int tally_sched_submit_be(tally_sched *s, uint32_t client, const tally_kernel_desc *kernel,
                          const tally_config *config, uint32_t flags) {
  if (!s || !kernel || client >= s->n_clients) return TALLY_ERR_INVALID_ARG;
  const KernelOps *ops;
  tally_dim3 g;
  int rc = check_desc(kernel, &ops, &g);
  if (rc) return rc;
  BeWork w;
  w.desc = *kernel;
  memcpy(w.args, kernel->args, ops->args_size);
  w.loop = (flags & TALLY_SUBMIT_LOOP) != 0;
  w.last_of_step = (flags & TALLY_SUBMIT_END_OF_STEP) != 0;
  if (config) {
    if (config->kind > 2 || (config->kind != 2 && config->param == 0)) return TALLY_ERR_INVALID_ARG;
    if (config->kind != 2 && !ops->transformable) return TALLY_ERR_UNSUPPORTED;
    if (config->kind == 0 && config->param > s->ctx->max_workers[kernel->kernel_id]) return TALLY_ERR_INVALID_ARG;
    w.config = *config;
  } else {
    if (!ops->transformable) return TALLY_ERR_UNSUPPORTED;
    w.config = tally_config{kCfgAuto, 0, 0, 0.f, 0.f};
  }
  {
    std::lock_guard<std::mutex> lk(s->mu);
    s->clients[client].queue.push_back(w);
  }
  s->cv.notify_all();
  return TALLY_OK;
}

int tally_sched_submit_hi(tally_sched *s, const tally_kernel_desc *kernels, uint32_t n) {
  if (!s || !kernels || n == 0) return TALLY_ERR_INVALID_ARG;
  if (s->hi_inflight) return TALLY_ERR_BAD_STATE;
  tally_ctx *ctx = s->ctx;
  uint32_t hl = 0, hw = 0, hr = 0;  // largest demand of one high-priority workgroup
  for (uint32_t i = 0; i < n; ++i) {
    const KernelOps *ops;
    tally_dim3 g;
    int rc = check_desc(&kernels[i], &ops, &g);
    if (rc) return rc;
    const uint32_t *ft = ctx->foot[kernels[i].kernel_id][1];
    hl = ft[0] > hl ? ft[0] : hl;
    hw = ft[1] > hw ? ft[1] : hw;
    const uint32_t per_simd = ((ft[1] + 3) / 4) * ft[2];
    hr = per_simd > hr ? per_simd : hr;
  }
  // the request time is published before the flag that makes the other thread read it
  s->t_preempt = now_us();
  s->hi_active = true;
  if (s->opts.policy == 0) {   // preempt_best_effort_kernel()
    for (uint32_t c = 0; c < s->n_clients; ++c) {
      BeClient &cl = s->clients[c];
      SpinGuard g(cl.lock);
      if (!cl.job || cl.job->kind != KIND_PTB) continue;
      // Workers may pause inside their blocks only if every kernel of the request fits
      // beside the paused workgroups on a compute unit; otherwise the request would wait
      // for them while they wait for it: then they give way at block boundaries only.
      const bool fits = cl.dl + hl <= ctx->lds_per_cu && cl.dw + hw <= 32u && cl.dr + hr <= 512u;
      if (fits && !(s->opts.flags & TALLY_SCHED_NO_PAUSE)) (void)tally_preempt_pausing(cl.job);
      else (void)tally_preempt(cl.job);
    }
  }
  int rc = TALLY_OK;
  for (uint32_t i = 0; i < n && rc == TALLY_OK; ++i) rc = tally_launch_native(ctx, &kernels[i], 1);
  if (rc == TALLY_OK) rc = tally_marker(ctx, 1, ++s->hi_seq);
  if (rc != TALLY_OK) { s->hi_active = false; return rc; }
  s->hi_inflight = true;
  return TALLY_OK;
}

int tally_sched_poll(tally_sched *s, int more_pending, int *hi_in_flight) {
  if (!s) return TALLY_ERR_INVALID_ARG;
  int rc = s->rc.load();
  if (rc) return rc;
  if (s->hi_inflight) {
    uint32_t seen;
    (void)tally_marker_read(s->ctx, 1, &seen);
    if (seen == s->hi_seq) {
      s->hi_inflight = false;
      s->hi_done++;
      // a queued request keeps the best-effort clients held; otherwise release them and
      // end the pause, so that workers pausing inside a block carry on at once
      if (!more_pending) {
        for (uint32_t c = 0; c < s->n_clients; ++c) {
          BeClient &cl = s->clients[c];
          SpinGuard g(cl.lock);
          if (cl.job) (void)tally_end_pause(cl.job);
        }
        s->hi_active = false;
      }
    }
  }
  if (hi_in_flight) *hi_in_flight = s->hi_inflight ? 1 : 0;
  return TALLY_OK;
}

int tally_sched_enable_be(tally_sched *s, int enable) {
  if (!s) return TALLY_ERR_INVALID_ARG;
  s->be_enabled = enable != 0;
  s->cv.notify_all();
  return TALLY_OK;
}

int tally_sched_stats(tally_sched *s, tally_sched_stats_t *out) {
  if (!s || !out) return TALLY_ERR_INVALID_ARG;
  memset(out, 0, sizeof(*out));
  out->hi_requests_done = s->hi_done;
  for (uint32_t c = 0; c < s->n_clients; ++c) {
    out->be_client_kernels_done[c] = s->clients[c].kernels_done.load();
    out->be_kernels_done += out->be_client_kernels_done[c];
  }
  out->be_steps_done = s->n_clients ? s->clients[0].steps_done.load() : 0;
  out->n_preempts = s->n_preempts.load();
  out->profile_samples = s->profile_samples.load();
  out->configs_fixed = s->configs_fixed.load();
  return TALLY_OK;
}

int tally_sched_take_preempt_latencies(tally_sched *s, double *out, uint32_t cap, uint32_t *n) {
  if (!s || !n || (cap && !out)) return TALLY_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(s->pre_mu);
  uint32_t k = (uint32_t)s->pre_ring.size();
  if (k > cap) k = cap;
  for (uint32_t i = 0; i < k; ++i) out[i] = s->pre_ring[i];
  s->pre_ring.erase(s->pre_ring.begin(), s->pre_ring.begin() + k);
  *n = k;
  return TALLY_OK;
}

// Replay driver: one fixed request at given arrival times against looping best-effort
// steps, on top of the scheduler above.
int tally_sched_run(tally_ctx *ctx, tally_sched_run_t *run) {
  if (!ctx || !run) return TALLY_ERR_INVALID_ARG;
  if (run->n_arrivals && (!run->arrivals_us || !run->latency_us || !run->hi_kernels ||
                          !run->n_hi_kernels))
    return TALLY_ERR_INVALID_ARG;
  if (run->n_be_items && !run->be_items) return TALLY_ERR_INVALID_ARG;
  if (run->policy > 2) return TALLY_ERR_INVALID_ARG;
  // validate every descriptor before anything is launched
  for (uint32_t i = 0; i < run->n_hi_kernels && run->n_arrivals; ++i) {
    const KernelOps *ops;
    tally_dim3 g;
    int rc = check_desc(&run->hi_kernels[i], &ops, &g);
    if (rc) return rc;
  }
  for (uint32_t i = 0; i < run->n_be_items; ++i) {
    if (!run->be_items[i].kernel || run->be_items[i].config.kind > kCfgAuto) return TALLY_ERR_INVALID_ARG;
    const KernelOps *ops;
    tally_dim3 g;
    int rc = check_desc(run->be_items[i].kernel, &ops, &g);
    if (rc) return rc;
  }
  // best-effort clients: one owning every item unless the caller splits them up
  uint32_t n_clients = run->n_be_items ? 1 : 0;
  if (run->n_be_items && run->n_be_clients) {
    if (!run->be_client_items || run->n_be_clients > (uint32_t)kMaxBeClients) return TALLY_ERR_INVALID_ARG;
    uint64_t sum = 0;
    for (uint32_t c = 0; c < run->n_be_clients; ++c) {
      if (run->be_client_items[c] == 0) return TALLY_ERR_INVALID_ARG;
      sum += run->be_client_items[c];
    }
    if (sum != run->n_be_items) return TALLY_ERR_INVALID_ARG;
    n_clients = run->n_be_clients;
  }
  tally_sched_opts opts;
  memset(&opts, 0, sizeof(opts));
  opts.policy = run->policy;
  opts.n_be_clients = n_clients;
  opts.threshold_ms = run->threshold_ms;
  opts.profile_runs = run->profile_runs;
  opts.flags = run->sched_flags;
  tally_sched *s = nullptr;
  int rc = tally_sched_create(ctx, &opts, &s);
  if (rc) return rc;
  (void)tally_sched_enable_be(s, 0);   // nothing starts before the clock does
  for (uint32_t c = 0, first = 0; c < n_clients && rc == TALLY_OK; ++c) {
    const uint32_t count = run->n_be_clients ? run->be_client_items[c] : run->n_be_items;
    for (uint32_t i = 0; i < count && rc == TALLY_OK; ++i) {
      const tally_be_item &it = run->be_items[first + i];
      rc = tally_sched_submit_be(s, c, it.kernel, it.config.kind == kCfgAuto ? nullptr : &it.config,
                                 TALLY_SUBMIT_LOOP | (i + 1 == count ? TALLY_SUBMIT_END_OF_STEP : 0u));
    }
    first += count;
  }
  if (rc) { (void)tally_sched_destroy(s); return rc; }

  run->n_preempts = 0;
  run->be_kernels_done = 0;
  run->be_steps_done = 0;
  const double last_arrival = run->n_arrivals ? run->arrivals_us[run->n_arrivals - 1] : 0.0;
  const double t_end = last_arrival + run->tail_us;
  const double t0 = now_us();
  const uint32_t toggle = run->n_arrivals ? run->be_toggle_every : 0;
  bool be_on = toggle == 0;
  double t_on = 0.0, enabled_us = 0.0;
  (void)tally_sched_enable_be(s, be_on ? 1 : 0);
  uint32_t next_arrival = 0, cur = 0, completed = 0;
  int inflight = 0;
  while (rc == TALLY_OK) {
    const double now = now_us() - t0;
    if (inflight) {
      const bool more = next_arrival < run->n_arrivals && run->arrivals_us[next_arrival] <= now;
      rc = tally_sched_poll(s, more ? 1 : 0, &inflight);
      if (rc) break;
      if (!inflight) {
        run->latency_us[cur] = (now_us() - t0) - run->arrivals_us[cur];
        completed++;
      }
    }
    if (toggle && !inflight && next_arrival < run->n_arrivals) {
      // switch the best-effort side for the block of arrivals that starts next, as soon as
      // the last request of the previous block is done
      const bool want_on = ((next_arrival / toggle) & 1u) != 0;
      if (want_on != be_on) {
        be_on = want_on;
        if (be_on) t_on = now; else enabled_us += now - t_on;
        (void)tally_sched_enable_be(s, be_on ? 1 : 0);
      }
    }
    if (!inflight && next_arrival < run->n_arrivals && run->arrivals_us[next_arrival] <= now) {
      cur = next_arrival++;
      rc = tally_sched_submit_hi(s, run->hi_kernels, run->n_hi_kernels);
      if (rc) break;
      if (run->issue_us) run->issue_us[cur] = (now_us() - t0) - run->arrivals_us[cur];
      inflight = 1;
    }
    if (!inflight && completed == run->n_arrivals && now >= t_end) break;
    if (!inflight && run->n_arrivals == 0) {
      int dummy;
      rc = tally_sched_poll(s, 0, &dummy);   // surfaces an error of the best-effort thread
    }
  }
  run->window_us = now_us() - t0;
  if (be_on) enabled_us += run->window_us - t_on;
  run->be_enabled_us = toggle ? enabled_us : run->window_us;
  tally_sched_stats_t st;
  (void)tally_sched_stats(s, &st);
  run->be_kernels_done = st.be_kernels_done;
  run->be_steps_done = st.be_steps_done;
  run->n_preempts = (uint32_t)st.n_preempts;
  run->profile_samples = st.profile_samples;
  run->configs_fixed = st.configs_fixed;
  if (run->be_client_kernels_done)
    for (uint32_t c = 0; c < n_clients; ++c) run->be_client_kernels_done[c] = st.be_client_kernels_done[c];
  if (run->preempt_latency_us && run->preempt_cap) {
    uint32_t got = 0;
    (void)tally_sched_take_preempt_latencies(s, run->preempt_latency_us, run->preempt_cap, &got);
  }
  int rc2 = tally_sched_destroy(s);   // drains and frees what is in flight; not part of the window
  return rc ? rc : rc2;
}

}  // extern "C"
