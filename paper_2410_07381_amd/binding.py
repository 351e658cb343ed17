"""Thin ctypes binding of libtally.so: argument marshalling only.

Every step of the path (the three launch forms, preemption, resume, profiling, the
scheduling loop) runs inside the library.  PyTorch appears only as the owner of
device memory and streams.  There is no CPU fallback: if the library is missing the
import fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

# Hardware queues.  HIP folds a process's streams onto GPU_MAX_HW_QUEUES hardware queues
# (4 unless the environment says otherwise) and reads the variable when it initialises;
# streams that share a queue run in order.  The scheduler needs one queue each for the
# high-priority stream, the best-effort stream and the relay stream beside the null
# stream's, and two more per further best-effort client (2 + 2n for n clients).  This
# module does not touch the environment: a program that wants several clients sets the
# variable itself before its first GPU call, and the library refuses a run whose clients
# would not get queues of their own.
def hw_queues():
    """The number of hardware queues this process asked HIP for (its default is 4)."""
    try:
        return int(os.environ.get("GPU_MAX_HW_QUEUES", "4"))
    except ValueError:
        return 4


_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtally.so")

# ---------------------------------------------------------------- enums
K_SAXPY, K_REDUCE_SUM, K_REDUCE_FINAL, K_GEMM_BF16, K_GEMV_BF16 = 0, 1, 2, 3, 4
K_SOFTMAX_F32, K_LAYERNORM_F32, K_ATTN_DECODE_BF16, K_GEMM_BF16_SMALL = 5, 6, 7, 8
K_GEMM_BF16_N128 = 9
JOB_QUEUED, JOB_RUNNING, JOB_STOPPED, JOB_COMPLETE = 0, 1, 2, 3
OK, ERR_INVALID_ARG, ERR_BAD_STATE, ERR_HIP, ERR_NOMEM, ERR_UNSUPPORTED = 0, -1, -2, -3, -4, -5
CFG_PTB, CFG_SLICED, CFG_NATIVE, CFG_AUTO = 0, 1, 2, 3
SUBMIT_LOOP, SUBMIT_END_OF_STEP = 1, 2
SCHED_NO_PAUSE = 1
POLICY_TALLY, POLICY_PRIORITY_NATIVE, POLICY_NONE = 0, 1, 2

EXPORTS = [
    "tally_create", "tally_destroy", "tally_logical_grid", "tally_attn_decode_scratch_bytes",
    "tally_launch_native", "tally_launch_sliced", "tally_launch_ptb", "tally_preempt",
    "tally_resume", "tally_progress", "tally_pump", "tally_wait", "tally_job_free",
    "tally_launch_ptb_until", "tally_resume_until", "tally_coverage", "tally_marker",
    "tally_marker_read", "tally_last_preempt_latency_us", "tally_last_hip_error",
    "tally_strerror", "tally_max_workers", "tally_kernel_footprint", "tally_mfma_ceiling_tflops", "tally_device_info", "tally_stream_report", "tally_ptb_turnaround_ms", "tally_select_config",
    "tally_profile", "tally_lookup_config", "tally_sched_run", "tally_set_yield_bound_us",
    "tally_launch_attn_decode_static", "tally_preempt_pausing", "tally_end_pause",
    "tally_candidate_configs", "tally_profile_table", "tally_profile_reset",
    "tally_sched_create", "tally_sched_destroy", "tally_sched_submit_be", "tally_sched_submit_hi",
    "tally_sched_poll", "tally_sched_enable_be", "tally_sched_stats",
    "tally_sched_take_preempt_latencies", "tally_set_yield_every",
]


class Dim3(C.Structure):
    _fields_ = [("x", C.c_uint32), ("y", C.c_uint32), ("z", C.c_uint32)]


class SaxpyArgs(C.Structure):
    _fields_ = [("x", C.c_void_p), ("y", C.c_void_p), ("a", C.c_float), ("n", C.c_uint32)]


class ReduceSumArgs(C.Structure):
    _fields_ = [("x", C.c_void_p), ("partial", C.c_void_p), ("n", C.c_uint64)]


class ReduceFinalArgs(C.Structure):
    _fields_ = [("partial", C.c_void_p), ("total", C.c_void_p), ("count", C.c_uint32)]


class GemmArgs(C.Structure):
    _fields_ = [("A", C.c_void_p), ("Bt", C.c_void_p), ("C", C.c_void_p),
                ("m", C.c_uint32), ("n", C.c_uint32), ("k", C.c_uint32), ("batch", C.c_uint32),
                ("stride_a", C.c_uint64), ("stride_b", C.c_uint64), ("stride_c", C.c_uint64),
                ("lda", C.c_uint32), ("ldb", C.c_uint32)]


class GemvArgs(C.Structure):
    _fields_ = [("x", C.c_void_p), ("W", C.c_void_p), ("y", C.c_void_p),
                ("n", C.c_uint32), ("k", C.c_uint32)]


class SoftmaxArgs(C.Structure):
    _fields_ = [("x", C.c_void_p), ("y", C.c_void_p), ("rows", C.c_uint32), ("cols", C.c_uint32)]


class LayerNormArgs(C.Structure):
    _fields_ = [("x", C.c_void_p), ("gamma", C.c_void_p), ("beta", C.c_void_p), ("y", C.c_void_p),
                ("rows", C.c_uint32), ("cols", C.c_uint32), ("eps", C.c_float)]


class AttnDecodeArgs(C.Structure):
    _fields_ = [("q", C.c_void_p), ("K", C.c_void_p), ("V", C.c_void_p), ("out", C.c_void_p),
                ("scratch", C.c_void_p), ("tokens", C.c_uint32), ("heads", C.c_uint32),
                ("dim", C.c_uint32)]


class KernelDesc(C.Structure):
    _fields_ = [("kernel_id", C.c_uint32), ("grid", Dim3), ("block", Dim3),
                ("args", C.c_void_p), ("args_size", C.c_size_t)]


class CoverRec(C.Structure):
    _fields_ = [("count", C.c_uint32), ("bx", C.c_uint32), ("by", C.c_uint32), ("bz", C.c_uint32),
                ("segment", C.c_uint32), ("worker", C.c_uint32)]


COVER_DTYPE = np.dtype([("count", "<u4"), ("bx", "<u4"), ("by", "<u4"), ("bz", "<u4"),
                        ("segment", "<u4"), ("worker", "<u4")])


class Config(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("param", C.c_uint32), ("chunk", C.c_uint32),
                ("latency_ms", C.c_float), ("turnaround_ms", C.c_float)]


class BeItem(C.Structure):
    _fields_ = [("kernel", C.POINTER(KernelDesc)), ("config", Config)]


class SchedRun(C.Structure):
    _fields_ = [("hi_kernels", C.POINTER(KernelDesc)), ("n_hi_kernels", C.c_uint32),
                ("arrivals_us", C.POINTER(C.c_double)), ("n_arrivals", C.c_uint32),
                ("be_items", C.POINTER(BeItem)), ("n_be_items", C.c_uint32),
                ("policy", C.c_uint32), ("tail_us", C.c_double),
                ("latency_us", C.POINTER(C.c_double)),
                ("preempt_latency_us", C.POINTER(C.c_double)), ("preempt_cap", C.c_uint32),
                ("n_preempts", C.c_uint32),
                ("be_kernels_done", C.c_uint64), ("be_steps_done", C.c_uint64),
                ("window_us", C.c_double), ("issue_us", C.POINTER(C.c_double)),
                ("be_client_items", C.POINTER(C.c_uint32)), ("n_be_clients", C.c_uint32),
                ("be_client_kernels_done", C.POINTER(C.c_uint64)),
                ("threshold_ms", C.c_double), ("profile_runs", C.c_uint32),
                ("sched_flags", C.c_uint32),
                ("profile_samples", C.c_uint64), ("configs_fixed", C.c_uint64),
                ("be_toggle_every", C.c_uint32), ("be_enabled_us", C.c_double)]


class SchedOpts(C.Structure):
    _fields_ = [("policy", C.c_uint32), ("n_be_clients", C.c_uint32), ("threshold_ms", C.c_double),
                ("profile_runs", C.c_uint32), ("flags", C.c_uint32)]


class SchedStats(C.Structure):
    _fields_ = [("hi_requests_done", C.c_uint64), ("be_kernels_done", C.c_uint64),
                ("be_steps_done", C.c_uint64), ("be_client_kernels_done", C.c_uint64 * 8),
                ("n_preempts", C.c_uint64), ("profile_samples", C.c_uint64),
                ("configs_fixed", C.c_uint64)]


class TallyError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = _lib.tally_strerror(status).decode() if _lib is not None else str(status)
        hip = _lib.tally_last_hip_error() if (_lib is not None and status == ERR_HIP) else 0
        super().__init__(f"{what}: {msg} (status {status}" + (f", hip error {hip})" if hip else ")"))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2410_07381_amd.build). "
            "There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    vp, u32, u64, i32, dbl = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int, C.c_double
    P = C.POINTER
    sig = {
        "tally_create": ([P(vp), vp, vp], i32),
        "tally_destroy": ([vp], i32),
        "tally_logical_grid": ([u32, vp, C.c_size_t, P(Dim3), P(Dim3)], i32),
        "tally_attn_decode_scratch_bytes": ([u32], C.c_size_t),
        "tally_launch_native": ([vp, P(KernelDesc), i32], i32),
        "tally_launch_attn_decode_static": ([vp, P(AttnDecodeArgs), i32], i32),
        "tally_launch_sliced": ([vp, P(KernelDesc), u32, u32, i32, P(vp)], i32),
        "tally_launch_ptb": ([vp, P(KernelDesc), u32, u32, i32, P(vp)], i32),
        "tally_preempt": ([vp], i32),
        "tally_resume": ([vp], i32),
        "tally_progress": ([vp, P(u64), P(u64), P(i32)], i32),
        "tally_pump": ([vp], i32),
        "tally_wait": ([vp, P(i32)], i32),
        "tally_job_free": ([vp], i32),
        "tally_launch_ptb_until": ([vp, P(KernelDesc), u32, u32, u64, i32, P(vp)], i32),
        "tally_resume_until": ([vp, u64], i32),
        "tally_coverage": ([vp, vp, C.c_size_t], i32),
        "tally_marker": ([vp, i32, u32], i32),
        "tally_marker_read": ([vp, i32, P(u32)], i32),
        "tally_last_preempt_latency_us": ([vp, P(dbl)], i32),
        "tally_last_hip_error": ([], i32),
        "tally_strerror": ([i32], C.c_char_p),
        "tally_device_info": ([P(u32), P(u32), P(u32)], i32),
        "tally_stream_report": ([vp, P(i32), P(u32)], i32),
        "tally_ptb_turnaround_ms": ([dbl, u32, u32, u64], dbl),
        "tally_select_config": ([P(Config), u32, dbl], i32),
        "tally_profile": ([vp, P(KernelDesc), P(Config), u32, u32, dbl, P(u32)], i32),
        "tally_lookup_config": ([vp, P(KernelDesc), P(Config)], i32),
        "tally_sched_run": ([vp, P(SchedRun)], i32),
        "tally_set_yield_bound_us": ([vp, u32], i32),
        "tally_max_workers": ([vp, P(KernelDesc), P(u32)], i32),
        "tally_kernel_footprint": ([vp, u32, i32, P(u32), P(u32), P(u32)], i32),
        "tally_mfma_ceiling_tflops": ([vp, u32, P(dbl)], i32),
        "tally_set_yield_every": ([vp, u32], i32),
        "tally_preempt_pausing": ([vp], i32),
        "tally_end_pause": ([vp], i32),
        "tally_candidate_configs": ([vp, P(KernelDesc), P(Config), u32, P(u32)], i32),
        "tally_profile_table": ([vp, P(KernelDesc), P(Config), u32, P(u32), P(u32), P(i32)], i32),
        "tally_profile_reset": ([vp], i32),
        "tally_sched_create": ([vp, P(SchedOpts), P(vp)], i32),
        "tally_sched_destroy": ([vp], i32),
        "tally_sched_submit_be": ([vp, u32, P(KernelDesc), P(Config), u32], i32),
        "tally_sched_submit_hi": ([vp, P(KernelDesc), u32], i32),
        "tally_sched_poll": ([vp, i32, P(i32)], i32),
        "tally_sched_enable_be": ([vp, i32], i32),
        "tally_sched_stats": ([vp, P(SchedStats)], i32),
        "tally_sched_take_preempt_latencies": ([vp, P(dbl), u32, P(u32)], i32),
    }
    assert set(sig) == set(EXPORTS), set(sig) ^ set(EXPORTS)
    for name, (argtypes, restype) in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = restype
    return lib


_lib = None
_lib = _load()


def lib():
    return _lib


def _check(rc, what):
    if rc != OK:
        raise TallyError(rc, what)


# ---------------------------------------------------------------- descriptors
_ARGS_FOR = {
    K_SAXPY: SaxpyArgs, K_REDUCE_SUM: ReduceSumArgs, K_REDUCE_FINAL: ReduceFinalArgs,
    K_GEMM_BF16: GemmArgs, K_GEMM_BF16_SMALL: GemmArgs, K_GEMM_BF16_N128: GemmArgs,
    K_GEMV_BF16: GemvArgs,
    K_SOFTMAX_F32: SoftmaxArgs, K_LAYERNORM_F32: LayerNormArgs, K_ATTN_DECODE_BF16: AttnDecodeArgs,
}


class Kernel:
    """A kernel descriptor plus the objects that must outlive it (args struct, tensors)."""

    def __init__(self, kernel_id, args, keep=()):
        assert isinstance(args, _ARGS_FOR[kernel_id])
        self.kernel_id = kernel_id
        self.args = args
        self.keep = tuple(keep)
        g, b = Dim3(), Dim3()
        _check(_lib.tally_logical_grid(kernel_id, C.addressof(args), C.sizeof(args),
                                       C.byref(g), C.byref(b)), "tally_logical_grid")
        self.desc = KernelDesc(kernel_id, g, b, C.addressof(args), C.sizeof(args))

    @property
    def grid(self):
        return (self.desc.grid.x, self.desc.grid.y, self.desc.grid.z)

    @property
    def total_blocks(self):
        g = self.grid
        return g[0] * g[1] * g[2]


def logical_grid(kernel_id, args):
    g, b = Dim3(), Dim3()
    _check(_lib.tally_logical_grid(kernel_id, C.addressof(args), C.sizeof(args), C.byref(g),
                                   C.byref(b)), "tally_logical_grid")
    return (g.x, g.y, g.z), (b.x, b.y, b.z)


def saxpy(x, y, a):
    return Kernel(K_SAXPY, SaxpyArgs(x.data_ptr(), y.data_ptr(), float(a), x.numel()), (x, y))


def reduce_sum(x, partial):
    return Kernel(K_REDUCE_SUM, ReduceSumArgs(x.data_ptr(), partial.data_ptr(), x.numel()),
                  (x, partial))


def reduce_final(partial, total, count=None):
    n = partial.numel() if count is None else count
    return Kernel(K_REDUCE_FINAL, ReduceFinalArgs(partial.data_ptr(), total.data_ptr(), n),
                  (partial, total))


def gemm_bf16(A, Bt, Cout, small=False, n128=False):
    """A [batch,m,k], Bt [batch,n,k], C [batch,m,n]; 16-bit storage tensors.  Tiles of
    256 x 256 outputs, 256 x 128 with n128, 32 x 32 (ragged edges allowed) with small.
    A and Bt may be views with padded rows (last dimension contiguous): their row and
    batch pitches are taken from the tensors; C must be contiguous."""
    batch, m, k = A.shape
    n = Bt.shape[1]
    assert A.stride(2) == 1 and Bt.stride(2) == 1 and Cout.is_contiguous()
    args = GemmArgs(A.data_ptr(), Bt.data_ptr(), Cout.data_ptr(), m, n, k, batch,
                    A.stride(0), Bt.stride(0), m * n, A.stride(1), Bt.stride(1))
    kid = K_GEMM_BF16_SMALL if small else (K_GEMM_BF16_N128 if n128 else K_GEMM_BF16)
    return Kernel(kid, args, (A, Bt, Cout))


def gemv_bf16(x, W, y):
    n, k = W.shape
    return Kernel(K_GEMV_BF16, GemvArgs(x.data_ptr(), W.data_ptr(), y.data_ptr(), n, k), (x, W, y))


def softmax_f32(x, y):
    rows, cols = x.shape
    return Kernel(K_SOFTMAX_F32, SoftmaxArgs(x.data_ptr(), y.data_ptr(), rows, cols), (x, y))


def layernorm_f32(x, gamma, beta, y, eps):
    rows, cols = x.shape
    return Kernel(K_LAYERNORM_F32,
                  LayerNormArgs(x.data_ptr(), gamma.data_ptr(), beta.data_ptr(), y.data_ptr(),
                                rows, cols, float(eps)), (x, gamma, beta, y))


def attn_decode_bf16(q, Kc, Vc, out, scratch):
    tokens, heads, dim = Kc.shape
    return Kernel(K_ATTN_DECODE_BF16,
                  AttnDecodeArgs(q.data_ptr(), Kc.data_ptr(), Vc.data_ptr(), out.data_ptr(),
                                 scratch.data_ptr(), tokens, heads, dim), (q, Kc, Vc, out, scratch))


def attn_decode_scratch_bytes(heads):
    return int(_lib.tally_attn_decode_scratch_bytes(heads))


# ---------------------------------------------------------------- context / jobs
class Job:
    def __init__(self, handle, kernel):
        self.h = handle
        self.kernel = kernel

    def preempt(self, pause=False):
        """Raise the preemption signal; with pause, also ask workers to pause inside long blocks."""
        if pause:
            _check(_lib.tally_preempt_pausing(self.h), "tally_preempt_pausing")
        else:
            _check(_lib.tally_preempt(self.h), "tally_preempt")

    def end_pause(self):
        _check(_lib.tally_end_pause(self.h), "tally_end_pause")

    def resume(self, stop_at=None):
        if stop_at is None:
            _check(_lib.tally_resume(self.h), "tally_resume")
        else:
            _check(_lib.tally_resume_until(self.h, int(stop_at)), "tally_resume_until")

    def progress(self):
        d, t, s = C.c_uint64(), C.c_uint64(), C.c_int()
        _check(_lib.tally_progress(self.h, C.byref(d), C.byref(t), C.byref(s)), "tally_progress")
        return d.value, t.value, s.value

    def pump(self):
        _check(_lib.tally_pump(self.h), "tally_pump")

    def wait(self):
        s = C.c_int()
        _check(_lib.tally_wait(self.h, C.byref(s)), "tally_wait")
        return s.value

    def coverage(self):
        rec = np.zeros(self.kernel.total_blocks, dtype=COVER_DTYPE)
        _check(_lib.tally_coverage(self.h, rec.ctypes.data, rec.nbytes), "tally_coverage")
        return rec

    def preempt_latency_us(self):
        v = C.c_double()
        _check(_lib.tally_last_preempt_latency_us(self.h, C.byref(v)), "preempt latency")
        return v.value

    def free(self):
        if self.h is not None:
            _check(_lib.tally_job_free(self.h), "tally_job_free")
            self.h = None


class Context:
    def __init__(self, stream_hi, stream_be):
        """stream_hi / stream_be: torch.cuda.Stream objects (default priority)."""
        self._streams = (stream_hi, stream_be)
        h = C.c_void_p()
        _check(_lib.tally_create(C.byref(h), C.c_void_p(stream_hi.cuda_stream),
                                 C.c_void_p(stream_be.cuda_stream)), "tally_create")
        self.h = h

    def close(self):
        if self.h is not None:
            _check(_lib.tally_destroy(self.h), "tally_destroy")
            self.h = None

    def launch_native(self, kernel, hi=False):
        _check(_lib.tally_launch_native(self.h, C.byref(kernel.desc), 1 if hi else 0),
               "tally_launch_native")

    def launch_attn_decode_static(self, q, Kc, Vc, out, hi=False):
        """Decode attention with the library's own static split records (allocates nothing)."""
        tokens, heads, dim = Kc.shape
        args = AttnDecodeArgs(q.data_ptr(), Kc.data_ptr(), Vc.data_ptr(), out.data_ptr(), None,
                              tokens, heads, dim)
        _check(_lib.tally_launch_attn_decode_static(self.h, C.byref(args), 1 if hi else 0),
               "tally_launch_attn_decode_static")

    def launch_sliced(self, kernel, slice_blocks, max_in_flight=1, coverage=False):
        j = C.c_void_p()
        _check(_lib.tally_launch_sliced(self.h, C.byref(kernel.desc), slice_blocks, max_in_flight,
                                        int(coverage), C.byref(j)), "tally_launch_sliced")
        return Job(j, kernel)

    def launch_ptb(self, kernel, workers, chunk=1, coverage=False, stop_at=None):
        j = C.c_void_p()
        if stop_at is None:
            _check(_lib.tally_launch_ptb(self.h, C.byref(kernel.desc), workers, chunk,
                                         int(coverage), C.byref(j)), "tally_launch_ptb")
        else:
            _check(_lib.tally_launch_ptb_until(self.h, C.byref(kernel.desc), workers, chunk,
                                               int(stop_at), int(coverage), C.byref(j)),
                   "tally_launch_ptb_until")
        return Job(j, kernel)

    def set_yield_bound_us(self, us):
        _check(_lib.tally_set_yield_bound_us(self.h, int(us)), "tally_set_yield_bound_us")

    def stream_report(self):
        """Whether the caller's best-effort stream delays the high-priority one, and how many
        streams the library created and set aside because they would."""
        a, b = C.c_int(), C.c_uint32()
        _check(_lib.tally_stream_report(self.h, C.byref(a), C.byref(b)), "tally_stream_report")
        return {"be_delays_hi": bool(a.value & 1), "crowded": bool(a.value & 2), "set_aside": b.value}

    def set_yield_every(self, steps):
        _check(_lib.tally_set_yield_every(self.h, int(steps)), "tally_set_yield_every")

    def marker(self, value, hi=True):
        _check(_lib.tally_marker(self.h, 1 if hi else 0, value), "tally_marker")

    def marker_read(self, hi=True):
        v = C.c_uint32()
        _check(_lib.tally_marker_read(self.h, 1 if hi else 0, C.byref(v)), "tally_marker_read")
        return v.value

    def profile(self, kernel, candidates, runs=10, threshold_ms=0.0316):
        """candidates: list of (kind, param, chunk).  Returns (list of dicts, chosen index)."""
        arr = (Config * len(candidates))(*[Config(k, p, c, 0.0, 0.0) for k, p, c in candidates])
        chosen = C.c_uint32()
        _check(_lib.tally_profile(self.h, C.byref(kernel.desc), arr, len(candidates), runs,
                                  threshold_ms, C.byref(chosen)), "tally_profile")
        out = [dict(kind=c.kind, param=c.param, chunk=c.chunk, latency_ms=c.latency_ms,
                    turnaround_ms=c.turnaround_ms) for c in arr]
        return out, chosen.value

    def candidate_configs(self, kernel, cap=64):
        """The Section 4.2 candidate set of a kernel as a list of (kind, param, chunk)."""
        arr = (Config * cap)()
        n = C.c_uint32()
        _check(_lib.tally_candidate_configs(self.h, C.byref(kernel.desc), arr, cap, C.byref(n)),
               "tally_candidate_configs")
        return [(arr[i].kind, arr[i].param, arr[i].chunk) for i in range(n.value)]

    def profile_table(self, kernel, cap=64):
        """(list of candidate dicts with their sample counts, index of the fixed choice or -1)."""
        arr = (Config * cap)()
        smp = (C.c_uint32 * cap)()
        n, chosen = C.c_uint32(), C.c_int()
        _check(_lib.tally_profile_table(self.h, C.byref(kernel.desc), arr, cap, C.byref(n), smp,
                                        C.byref(chosen)), "tally_profile_table")
        rows = [dict(kind=arr[i].kind, param=arr[i].param, chunk=arr[i].chunk,
                     latency_ms=arr[i].latency_ms, turnaround_ms=arr[i].turnaround_ms,
                     samples=smp[i]) for i in range(min(n.value, cap))]
        return rows, chosen.value

    def profile_reset(self):
        _check(_lib.tally_profile_reset(self.h), "tally_profile_reset")

    def scheduler(self, policy=POLICY_TALLY, be_clients=1, threshold_ms=0.0, profile_runs=0, flags=0):
        return Scheduler(self, policy, be_clients, threshold_ms, profile_runs, flags)

    def mfma_ceiling_tflops(self, reps=10):
        """Measured bf16 matrix-pipe ceiling (register-only MFMA loop on every compute unit)."""
        v = C.c_double()
        _check(_lib.tally_mfma_ceiling_tflops(self.h, reps, C.byref(v)), "tally_mfma_ceiling_tflops")
        return v.value

    def kernel_footprint(self, kernel_id, form):
        """(LDS bytes, waves, registers per lane) of one workgroup; form 0 = persistent
        workers, 1 = original form."""
        a, b, c = C.c_uint32(), C.c_uint32(), C.c_uint32()
        _check(_lib.tally_kernel_footprint(self.h, kernel_id, form, C.byref(a), C.byref(b), C.byref(c)),
               "tally_kernel_footprint")
        return a.value, b.value, c.value

    def max_workers(self, kernel):
        """Largest worker count whose workgroups are all resident at once."""
        n = C.c_uint32()
        _check(_lib.tally_max_workers(self.h, C.byref(kernel.desc), C.byref(n)), "tally_max_workers")
        return n.value

    def lookup_config(self, kernel):
        c = Config()
        rc = _lib.tally_lookup_config(self.h, C.byref(kernel.desc), C.byref(c))
        if rc == ERR_BAD_STATE:
            return None
        _check(rc, "tally_lookup_config")
        return dict(kind=c.kind, param=c.param, chunk=c.chunk, latency_ms=c.latency_ms,
                    turnaround_ms=c.turnaround_ms)

    def sched_run(self, hi_kernels, arrivals_us, be_items, policy=POLICY_TALLY, tail_us=0.0,
                  be_clients=None, threshold_ms=0.0, profile_runs=0, flags=0, be_toggle_every=0):
        """hi_kernels: list of Kernel (one request).  be_items: list of (Kernel, (kind, param,
        chunk)).  be_clients: optional list of item counts, one per best-effort client (the
        items are the concatenation of the clients' steps).  Returns a dict of numpy arrays
        and counters."""
        n_hi = len(hi_kernels)
        hi_arr = (KernelDesc * max(n_hi, 1))(*[k.desc for k in hi_kernels])
        arrivals = np.ascontiguousarray(arrivals_us, dtype=np.float64)
        lat = np.zeros(len(arrivals), dtype=np.float64)
        cap = max(len(arrivals), 1)
        pre = np.zeros(cap, dtype=np.float64)
        items = (BeItem * max(len(be_items), 1))()
        for i, (k, cfg) in enumerate(be_items):
            items[i].kernel = C.pointer(k.desc)
            items[i].config = Config(cfg[0], cfg[1], cfg[2] if len(cfg) > 2 else 1, 0.0, 0.0)
        run = SchedRun()
        run.hi_kernels = hi_arr
        run.n_hi_kernels = n_hi
        run.arrivals_us = arrivals.ctypes.data_as(C.POINTER(C.c_double))
        run.n_arrivals = len(arrivals)
        run.be_items = items
        run.n_be_items = len(be_items)
        run.policy = policy
        run.tail_us = float(tail_us)
        run.threshold_ms = float(threshold_ms)
        run.profile_runs = int(profile_runs)
        run.sched_flags = int(flags)
        run.be_toggle_every = int(be_toggle_every)
        run.latency_us = lat.ctypes.data_as(C.POINTER(C.c_double))
        run.preempt_latency_us = pre.ctypes.data_as(C.POINTER(C.c_double))
        run.preempt_cap = cap
        per_client = None
        if be_clients is not None:
            counts = (C.c_uint32 * len(be_clients))(*be_clients)
            per_client = np.zeros(len(be_clients), dtype=np.uint64)
            run.be_client_items = counts
            run.n_be_clients = len(be_clients)
            run.be_client_kernels_done = per_client.ctypes.data_as(C.POINTER(C.c_uint64))
        issue = np.zeros(len(arrivals), dtype=np.float64)
        run.issue_us = issue.ctypes.data_as(C.POINTER(C.c_double))
        _check(_lib.tally_sched_run(self.h, C.byref(run)), "tally_sched_run")
        return {
            "latency_us": lat,
            "issue_us": issue,
            "preempt_latency_us": pre[: min(run.n_preempts, cap)].copy(),
            "n_preempts": run.n_preempts,
            "be_kernels_done": run.be_kernels_done,
            "be_steps_done": run.be_steps_done,
            "window_us": run.window_us,
            "be_client_kernels_done": per_client,
            "be_enabled_us": run.be_enabled_us,
            "profile_samples": run.profile_samples,
            "configs_fixed": run.configs_fixed,
        }


class Scheduler:
    """The priority scheduler as a running service (tally_sched_*)."""

    def __init__(self, ctx, policy, be_clients, threshold_ms, profile_runs, flags):
        self.ctx = ctx
        self._keep = []
        opts = SchedOpts(policy, be_clients, float(threshold_ms), int(profile_runs), int(flags))
        h = C.c_void_p()
        _check(_lib.tally_sched_create(ctx.h, C.byref(opts), C.byref(h)), "tally_sched_create")
        self.h = h

    def submit_be(self, kernel, config=None, client=0, loop=False, end_of_step=False):
        self._keep.append(kernel)
        cfg = None
        if config is not None:
            cfg = C.byref(Config(config[0], config[1], config[2] if len(config) > 2 else 1, 0.0, 0.0))
        flags = (SUBMIT_LOOP if loop else 0) | (SUBMIT_END_OF_STEP if end_of_step else 0)
        _check(_lib.tally_sched_submit_be(self.h, client, C.byref(kernel.desc), cfg, flags),
               "tally_sched_submit_be")

    def submit_hi(self, kernels):
        arr = (KernelDesc * len(kernels))(*[k.desc for k in kernels])
        _check(_lib.tally_sched_submit_hi(self.h, arr, len(kernels)), "tally_sched_submit_hi")

    def poll(self, more_pending=False):
        """True while the high-priority request is still in flight."""
        f = C.c_int()
        _check(_lib.tally_sched_poll(self.h, 1 if more_pending else 0, C.byref(f)), "tally_sched_poll")
        return bool(f.value)

    def enable_be(self, on=True):
        _check(_lib.tally_sched_enable_be(self.h, 1 if on else 0), "tally_sched_enable_be")

    def stats(self):
        st = SchedStats()
        _check(_lib.tally_sched_stats(self.h, C.byref(st)), "tally_sched_stats")
        return {"hi_requests_done": st.hi_requests_done, "be_kernels_done": st.be_kernels_done,
                "be_steps_done": st.be_steps_done,
                "be_client_kernels_done": list(st.be_client_kernels_done),
                "n_preempts": st.n_preempts, "profile_samples": st.profile_samples,
                "configs_fixed": st.configs_fixed}

    def take_preempt_latencies(self, cap=4096):
        buf = (C.c_double * cap)()
        n = C.c_uint32()
        _check(_lib.tally_sched_take_preempt_latencies(self.h, buf, cap, C.byref(n)),
               "tally_sched_take_preempt_latencies")
        return np.array(buf[: n.value], dtype=np.float64)

    def close(self):
        if self.h is not None:
            h, self.h = self.h, None
            _check(_lib.tally_sched_destroy(h), "tally_sched_destroy")


def device_info():
    a, b, c = C.c_uint32(), C.c_uint32(), C.c_uint32()
    _check(_lib.tally_device_info(C.byref(a), C.byref(b), C.byref(c)), "tally_device_info")
    return {"num_cus": a.value, "lds_bytes_per_cu": b.value, "wave_size": c.value}


def ptb_turnaround_ms(latency_ms, workers, chunk, total):
    return _lib.tally_ptb_turnaround_ms(latency_ms, workers, chunk, total)


def select_config(cands, threshold_ms=0.0316):
    """cands: list of dicts with kind, param, latency_ms, turnaround_ms (chunk optional)."""
    arr = (Config * len(cands))(*[Config(c["kind"], c["param"], c.get("chunk", 1),
                                         c["latency_ms"], c["turnaround_ms"]) for c in cands])
    return _lib.tally_select_config(arr, len(cands), threshold_ms)
