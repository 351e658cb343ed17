"""GPU parity: block coverage and indexing of the three launch forms against the oracle,
bit for bit, plus SAXPY / reduction outputs; all calls go through the C ABI."""
import time

import numpy as np
import pytest

import tally_inputs as TI
from oracle import kernels as OK
from oracle import schedules as OS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2410_07381_amd.binding as B
    assert torch.cuda.is_available(), "these tests need the MI355X"
    hi, be = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(hi, be)
    yield B, ctx, torch
    ctx.close()


def _saxpy_oracle(base, runner):
    a = dict(base, y=base["y"].copy())
    cov = runner(a)
    return a["y"], cov


# ------------------------------------------------------------------ configuration 0
def test_cfg0_saxpy_ptb_three_preemptions(env):
    """N = 2^20, grid 4096 x 256, 256 workers, 3 preemptions at seeded counter values,
    each followed by a resume."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_close_rel
    base = TI.saxpy_inputs(n=1 << 20, config_index=0)
    grid = OK.grid_of("saxpy", base)
    assert grid == (4096, 1, 1)
    pts = TI.preempt_points(4096, 3, config_index=0)
    assert len(pts) == 3 and all(1 <= p <= 4095 for p in pts)

    x, y = dev(base["x"]), dev(base["y"])
    torch.cuda.synchronize()
    k = B.saxpy(x, y, base["a"])
    assert k.grid == grid
    job = ctx.launch_ptb(k, 256, coverage=True, stop_at=pts[0])
    seen = []
    for nxt in pts[1:] + [None]:
        st = job.wait()
        done, total, _ = job.progress()
        seen.append(done)
        assert st == B.JOB_STOPPED and total == 4096
        job.resume(stop_at=nxt)
    assert job.wait() == B.JOB_COMPLETE
    assert seen == pts and job.progress()[0] == 4096
    rec = job.coverage()
    job.free()

    want_y, (cov, log) = _saxpy_oracle(
        base, lambda a: OS.run_ptb("saxpy", grid, a, 256, preempt_points=pts, seed=0))
    assert log == pts + [4096]
    assert_cover_equal(rec, cov)
    assert (rec["worker"] < 256).all()
    assert_close_rel(host(y), want_y, 1e-6)


@pytest.mark.parametrize("n,workers,chunk,pts", [
    (5000, 4, 1, [3, 11]),          # ragged last block
    (5000, 7, 3, [1, 19]),          # chunked fetch, stop inside a chunk
    (256 * 33, 64, 1, [10]),        # more workers than blocks
    (1000, 2, 1, []),
])
def test_saxpy_ptb_small(env, n, workers, chunk, pts):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_close_rel
    base = TI.saxpy_inputs(n=n, config_index=0)
    grid = OK.grid_of("saxpy", base)
    x, y = dev(base["x"]), dev(base["y"])
    torch.cuda.synchronize()
    k = B.saxpy(x, y, base["a"])
    stops = pts + [None]
    job = ctx.launch_ptb(k, workers, chunk=chunk, coverage=True, stop_at=stops[0])
    for nxt in stops[1:]:
        assert job.wait() == B.JOB_STOPPED
        job.resume(stop_at=nxt)
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    want_y, (cov, _) = _saxpy_oracle(
        base, lambda a: OS.run_ptb("saxpy", grid, a, workers, preempt_points=pts, seed=1))
    assert_cover_equal(rec, cov)
    assert_close_rel(host(y), want_y, 1e-6)


def test_degenerate_schedules(env):
    """A zero-block segment (preempted before the first fetch), one worker, a chunk and a
    slice larger than the whole grid, an empty input."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_close_rel
    base = TI.saxpy_inputs(n=256 * 7 + 3, config_index=0)          # 8 blocks
    grid = OK.grid_of("saxpy", base)
    want_y, (cov0, _) = _saxpy_oracle(base, lambda a: OS.run_ptb("saxpy", grid, a, 1, preempt_points=[], seed=0))

    def fresh():
        x, y = dev(base["x"]), dev(base["y"])
        torch.cuda.synchronize()
        return B.saxpy(x, y, base["a"]), y

    k, y = fresh()                                                  # stop before anything ran
    job = ctx.launch_ptb(k, 4, coverage=True, stop_at=0)
    assert job.wait() == B.JOB_STOPPED and job.progress()[0] == 0
    assert (job.coverage()["count"] == 0).all()
    job.resume()
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    assert (rec["count"] == 1).all() and (rec["segment"] == 1).all()
    assert_close_rel(host(y), want_y, 1e-6)

    k, y = fresh()                                                  # one worker, in order
    job = ctx.launch_ptb(k, 1, coverage=True)
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    assert_cover_equal(rec, cov0)
    assert (rec["worker"] == 0).all()
    assert_close_rel(host(y), want_y, 1e-6)

    k, y = fresh()                                                  # one fetch takes the grid
    job = ctx.launch_ptb(k, 3, chunk=1000, coverage=True)
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    assert (rec["count"] == 1).all() and len(set(rec["worker"].tolist())) == 1
    assert_close_rel(host(y), want_y, 1e-6)

    k, y = fresh()                                                  # one slice takes the grid
    job = ctx.launch_sliced(k, 1000, coverage=True)
    assert job.wait() == B.JOB_COMPLETE
    assert (job.coverage()["count"] == 1).all()
    job.free()
    assert_close_rel(host(y), want_y, 1e-6)

    empty = torch.zeros(0, device="cuda")
    with pytest.raises(B.TallyError):
        B.saxpy(empty, empty, 1.0)


def test_saxpy_native_and_sliced(env):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_close_rel
    base = TI.saxpy_inputs(n=256 * 16, config_index=0)        # the paper's 16-block example
    grid = OK.grid_of("saxpy", base)
    x, y = dev(base["x"]), dev(base["y"])
    y2 = dev(base["y"])
    torch.cuda.synchronize()
    job = ctx.launch_sliced(B.saxpy(x, y, base["a"]), 4, coverage=True)
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    want_y, (cov, _) = _saxpy_oracle(base, lambda a: OS.run_sliced("saxpy", grid, a, 4))
    assert_cover_equal(rec, cov)
    assert rec["bx"][4:8].tolist() == [4, 5, 6, 7]             # sub-kernel 2: offset 4
    assert_close_rel(host(y), want_y, 1e-6)
    ctx.launch_native(B.saxpy(x, y2, base["a"]))
    torch.cuda.synchronize()
    assert (host(y2).view(np.uint32) == host(y).view(np.uint32)).all()


@pytest.mark.parametrize("in_flight", [2, 3, 8])
def test_sliced_several_slices_in_flight(env, in_flight):
    """More than one sub-kernel enqueued at a time (the paper enqueues one): coverage and
    results are those of the one-at-a-time schedule, and a preemption drains every slice
    that was already enqueued before the job reports STOPPED."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_close_rel
    base = TI.saxpy_inputs(n=256 * 33 + 17, config_index=0)        # 34 blocks, ragged tail
    grid = OK.grid_of("saxpy", base)
    x, y = dev(base["x"]), dev(base["y"])
    torch.cuda.synchronize()
    job = ctx.launch_sliced(B.saxpy(x, y, base["a"]), 5, max_in_flight=in_flight, coverage=True)
    job.preempt()
    all_enqueued = 5 * in_flight >= 34                             # then nothing is left to stop
    assert job.wait() == (B.JOB_COMPLETE if all_enqueued else B.JOB_STOPPED)
    done = job.progress()[0]
    assert done == min(5 * in_flight, 34)                          # exactly the enqueued slices
    job.resume()                                                   # no-op on a complete job
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    first = min(in_flight, 7)                                      # slices before the preemption
    want_y, (cov, resumes) = _saxpy_oracle(
        base, lambda a: OS.run_sliced("saxpy", grid, a, 5, preempt_after_slices=[first]))
    assert resumes == ([] if all_enqueued else [done])
    assert_cover_equal(rec, cov)
    assert_close_rel(host(y), want_y, 1e-6)


def test_sliced_preempt_and_resume_segments(env):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_close_rel
    base = TI.saxpy_inputs(n=256 * 10, config_index=0)
    grid = OK.grid_of("saxpy", base)
    x, y = dev(base["x"]), dev(base["y"])
    torch.cuda.synchronize()
    job = ctx.launch_sliced(B.saxpy(x, y, base["a"]), 4, coverage=True)
    job.preempt()                        # first slice is already enqueued and will finish
    assert job.wait() == B.JOB_STOPPED
    assert job.progress()[0] == 4
    job.preempt()                        # no-op on a stopped job
    job.resume()
    job.preempt()
    assert job.wait() == B.JOB_STOPPED and job.progress()[0] == 8
    job.resume()
    assert job.wait() == B.JOB_COMPLETE
    job.resume()                         # no-op on a complete job
    rec = job.coverage()
    job.free()
    want_y, (cov, resumes) = _saxpy_oracle(
        base, lambda a: OS.run_sliced("saxpy", grid, a, 4, preempt_after_slices=[1, 2]))
    assert resumes == [4, 8]
    assert_cover_equal(rec, cov)
    assert_close_rel(host(y), want_y, 1e-6)


# ------------------------------------------------------------------ multi-dimensional grid
def test_ptb_three_dimensional_grid_mapping(env):
    """Batched 32-wide GEMM tiles give a (gx, gy, gz) grid: the rebuilt block indices
    must follow x-fastest order in both transformed forms."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_bf16_close
    g = TI.gemm_inputs(m=150, n=200, k=64, config_index=1, batch=3)
    a = dict(g, C=np.zeros((3, 150, 200), np.uint16))
    grid = OK.grid_of("gemm_bf16_small", a)
    assert grid == (7, 5, 3)
    A, Bt = dev(g["A"]), dev(g["Bt"])
    Cp, Cs = dev(a["C"]), dev(a["C"])
    torch.cuda.synchronize()
    job = ctx.launch_ptb(B.gemm_bf16(A, Bt, Cp, small=True), 5, coverage=True, stop_at=17)
    assert job.wait() == B.JOB_STOPPED
    job.resume()
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    cov, _ = OS.run_ptb("gemm_bf16_small", grid, a, 5, preempt_points=[17], seed=4)
    assert_cover_equal(rec, cov)
    assert_bf16_close(host(Cp), a["C"])
    job = ctx.launch_sliced(B.gemm_bf16(A, Bt, Cs, small=True), 7, coverage=True)
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    b = dict(g, C=np.zeros((3, 150, 200), np.uint16))
    cov, _ = OS.run_sliced("gemm_bf16_small", grid, b, 7)
    assert_cover_equal(rec, cov)
    assert (host(Cs) == host(Cp)).all()


# ------------------------------------------------------------------ asynchronous preemption
@pytest.mark.parametrize("workers,chunk", [(256, 1), (512, 8)])
def test_async_flag_preemption_prefix_and_exactly_once(env, workers, chunk):
    """Raise the real flag from the host while workers run.  The observed progress value is
    fed to the oracle as its preemption point; at the drain exactly the prefix has run."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal
    n = 1 << 28
    x = torch.rand(n, device="cuda")
    nb = n // 4096
    partial = torch.zeros(nb, device="cuda")
    torch.cuda.synchronize()
    k = B.reduce_sum(x, partial)
    pts = []
    job = ctx.launch_ptb(k, workers, chunk=chunk, coverage=True)
    for attempt in range(3):
        time.sleep(0.0001 if chunk == 1 else 0.00004)
        job.preempt()
        st = job.wait()
        done, total, _ = job.progress()
        if st == B.JOB_COMPLETE:
            break
        assert st == B.JOB_STOPPED and 0 <= done < total and done % chunk == 0
        lat = job.preempt_latency_us()
        assert 0 < lat < 5e4
        rec = job.coverage()
        assert (rec["count"][:done] == 1).all() and (rec["count"][done:] == 0).all()
        pts.append(done)
        job.resume()
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    assert len(pts) >= 1, "the kernel finished before any preemption landed"
    cov, log = OS.run_ptb(None, (nb, 1, 1), {}, workers, preempt_points=pts, seed=7, chunk=chunk)
    assert log == pts + [nb]
    assert_cover_equal(rec, cov)
    from gpu_util import oracle_block_sums, assert_close_rel
    sample = [0, nb - 1] + [int(v) for v in np.random.default_rng(3).integers(nb, size=1500)]
    idx, want = oracle_block_sums(host(x), sample)
    assert_close_rel(host(partial)[idx], want, 2e-6)


def test_many_preemptions_in_a_row_keep_exactly_once(env):
    """Sixty asynchronous preempt / drain / resume cycles on one job: the task counter is
    never reset (the base moves after every drain, the word accumulates every failed fetch
    and 2^31 per request, wrapping several times), yet every block runs exactly once, each
    drain leaves a prefix, and the segments are the ones the oracle gets from the same
    progress values."""
    B, ctx, torch = env
    from gpu_util import host, assert_cover_equal, oracle_block_sums, assert_close_rel
    n = 1 << 28
    x = torch.rand(n, device="cuda")
    nb = n // 4096
    partial = torch.zeros(nb, device="cuda")
    torch.cuda.synchronize()
    k = B.reduce_sum(x, partial)
    workers, chunk = 256, 4                      # slow enough (about 0.3 ms alone) to be caught
    pts = []
    job = ctx.launch_ptb(k, workers, chunk=chunk, coverage=True)
    for cycle in range(60):
        job.preempt()
        st = job.wait()
        done = job.progress()[0]
        if st == B.JOB_COMPLETE:
            break
        assert st == B.JOB_STOPPED and done % chunk == 0 and (not pts or done >= pts[-1])
        pts.append(done)
        job.resume()
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    assert len(pts) >= 10, pts
    assert (rec["count"] == 1).all()
    # (a request that found nothing new to stop repeats the progress value: an empty segment,
    # on the GPU and in the oracle alike)
    cov, log = OS.run_ptb(None, (nb, 1, 1), {}, workers, preempt_points=pts, seed=9, chunk=chunk)
    assert log == pts + [nb]
    assert_cover_equal(rec, cov)
    sample = [0, nb - 1] + [int(v) for v in np.random.default_rng(5).integers(nb, size=500)]
    idx, want = oracle_block_sums(host(x), sample)
    assert_close_rel(host(partial)[idx], want, 2e-6)


def test_preemption_reaches_workers_that_fill_the_gpu(env):
    """The largest worker count of the softmax kernel leaves no register free on any compute
    unit: the flag must still reach the workers (the relay is resident before them) and the
    job must drain long before it would have finished."""
    import time
    B, ctx, torch = env
    from gpu_util import host
    x = torch.randn((65536, 2048), device="cuda")
    y = torch.zeros_like(x)
    torch.cuda.synchronize()
    k = B.softmax_f32(x, y)
    w = ctx.max_workers(k)
    job = ctx.launch_ptb(k, w, chunk=2)
    t0 = time.perf_counter()
    while job.progress()[0] < 64 and time.perf_counter() - t0 < 1.0:
        pass
    job.preempt()
    assert job.wait() == B.JOB_STOPPED
    done, total, _ = job.progress()
    assert 0 < done < total // 2, (done, total)          # the whole kernel takes ~1.5 ms
    job.resume()
    assert job.wait() == B.JOB_COMPLETE
    job.free()
    torch.cuda.synchronize()
    from gpu_util import oracle_softmax_rows, assert_close_rel
    assert_close_rel(host(y)[::4099], oracle_softmax_rows(host(x)[::4099]), 1e-5, 1e-7)


# ------------------------------------------------------------------ reduction, configuration 2 shape
@pytest.mark.parametrize("slice_blocks", [1, 8, 64])
def test_reduce_sliced_ragged(env, slice_blocks):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_cover_equal, assert_close_rel
    n = 4096 * 37 + 123
    xs = TI.reduce_inputs(n=n, config_index=2)["x"]
    nb = OK.grid_of("reduce_sum", {"n": n})[0]
    x, partial, total = dev(xs), dev(np.zeros(nb, np.float32)), dev(np.zeros(1, np.float64))
    torch.cuda.synchronize()
    job = ctx.launch_sliced(B.reduce_sum(x, partial), slice_blocks, coverage=True)
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    ctx.launch_native(B.reduce_final(partial, total))
    torch.cuda.synchronize()
    a = {"x": xs, "n": n, "partial": np.zeros(nb, np.float32)}
    cov, _ = OS.run_sliced("reduce_sum", (nb, 1, 1), a, slice_blocks)
    assert_cover_equal(rec, cov)
    assert_close_rel(host(partial), a["partial"], 2e-6)
    f = {"partial": a["partial"], "count": nb, "total": np.zeros(1, np.float64)}
    OS.run_native("reduce_final", (1, 1, 1), f)
    assert_close_rel(host(total), f["total"], 1e-6)


def test_reduce_all_ones_exact_all_forms(env):
    B, ctx, torch = env
    from gpu_util import host
    n = 1 << 22
    x = torch.ones(n, device="cuda")
    for form in ("native", "sliced", "ptb", "ptb_chunk"):
        partial = torch.zeros(n // 4096, device="cuda")
        total = torch.zeros(1, device="cuda", dtype=torch.float64)
        torch.cuda.synchronize()
        k = B.reduce_sum(x, partial)
        if form == "native":
            ctx.launch_native(k)
        else:
            job = (ctx.launch_sliced(k, 100) if form == "sliced" else
                   ctx.launch_ptb(k, 512, chunk=4 if form == "ptb_chunk" else 1))
            assert job.wait() == B.JOB_COMPLETE
            job.free()
        ctx.launch_native(B.reduce_final(partial, total))
        torch.cuda.synchronize()
        assert (host(partial) == 4096.0).all(), form
        assert host(total)[0] == float(n), form


# ------------------------------------------------------------------ error behaviour
def test_error_paths(env):
    B, ctx, torch = env
    import ctypes as C
    x = torch.zeros(1024, device="cuda")
    y = torch.zeros(1024, device="cuda")
    k = B.saxpy(x, y, 1.0)
    lib = B.lib()
    j = C.c_void_p()
    assert lib.tally_launch_sliced(ctx.h, C.byref(k.desc), 0, 1, 0, C.byref(j)) == B.ERR_INVALID_ARG
    assert lib.tally_launch_ptb(ctx.h, C.byref(k.desc), 0, 1, 0, C.byref(j)) == B.ERR_INVALID_ARG
    assert lib.tally_launch_ptb(ctx.h, C.byref(k.desc), 4, 0, 0, C.byref(j)) == B.ERR_INVALID_ARG
    # more workers than are resident at once: the kernel could not be preempted promptly
    mw = ctx.max_workers(k)
    assert mw >= B.device_info()["num_cus"] and mw % B.device_info()["num_cus"] == 0
    assert lib.tally_launch_ptb(ctx.h, C.byref(k.desc), mw + 1, 1, 0, C.byref(j)) == B.ERR_INVALID_ARG
    bad = B.KernelDesc(k.desc.kernel_id, k.desc.grid, k.desc.block, k.desc.args, k.desc.args_size)
    bad.grid.x += 1                                     # not the kernel's logical grid
    assert lib.tally_launch_native(ctx.h, C.byref(bad), 0) == B.ERR_INVALID_ARG
    bad.grid.x -= 1
    bad.kernel_id = 99
    assert lib.tally_launch_native(ctx.h, C.byref(bad), 0) == B.ERR_INVALID_ARG
    bad.kernel_id = k.desc.kernel_id
    bad.args_size -= 4
    assert lib.tally_launch_native(ctx.h, C.byref(bad), 0) == B.ERR_INVALID_ARG
    assert lib.tally_preempt(None) == B.ERR_INVALID_ARG
    # decode attention is a two-phase kernel: only the original form exists
    q = torch.zeros((2, 128), dtype=torch.int16, device="cuda")
    kv = torch.zeros((64, 2, 128), dtype=torch.int16, device="cuda")
    out = torch.zeros((2, 128), dtype=torch.int16, device="cuda")
    scratch = torch.zeros(B.attn_decode_scratch_bytes(2), dtype=torch.uint8, device="cuda")
    ka = B.attn_decode_bf16(q, kv, kv, out, scratch)
    assert lib.tally_launch_ptb(ctx.h, C.byref(ka.desc), 4, 1, 0, C.byref(j)) == B.ERR_UNSUPPORTED
    assert lib.tally_launch_sliced(ctx.h, C.byref(ka.desc), 4, 1, 0, C.byref(j)) == B.ERR_UNSUPPORTED
    with pytest.raises(B.TallyError):
        ctx.max_workers(ka)
    # state machine: resume of a complete job and preempt of a complete job are no-ops
    job = ctx.launch_ptb(k, 2)
    assert job.wait() == B.JOB_COMPLETE
    job.preempt()
    job.resume()
    assert job.progress()[2] == B.JOB_COMPLETE
    job.free()
    torch.cuda.synchronize()
