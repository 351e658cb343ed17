"""Helpers for the GPU parity tests: device buffers from seeded host arrays, oracle runs
on copies of the same bits, and the comparison rules.

Tolerances (each follows from the arithmetic named beside it):
  fp32 elementwise (SAXPY)      1e-6 relative (one fused multiply-add vs fp64 rounded once)
  fp32 block sums               2e-6 relative (at most 23 fp32 roundings of 2^-24 each)
  softmax / LayerNorm           1e-5 relative + 1e-7 absolute (exp / rsqrt + reduction order)
  bf16 GEMM / GEMV / attention  |d| <= 1e-2 * max(|ref|, rms(ref)) and Frobenius 1e-2
"""
import numpy as np
import torch

from oracle import bf16 as obf16
from oracle import kernels as OK
from oracle import schedules as OS


def dev(arr):
    """Host numpy array -> device tensor holding the same bits."""
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def host(t):
    a = t.detach().cpu().numpy()
    if a.dtype == np.int16:
        return a.view(np.uint16)
    return a


def assert_cover_equal(rec, cov, check_segment=True):
    """Bit-exact comparison of GPU coverage records with the oracle's."""
    assert (rec["count"] == cov.count).all(), "block execution counts differ"
    assert (rec["bx"] == cov.bidx[:, 0]).all()
    assert (rec["by"] == cov.bidx[:, 1]).all()
    assert (rec["bz"] == cov.bidx[:, 2]).all()
    if check_segment:
        assert (rec["segment"] == cov.segment).all(), "launch segments differ"


def assert_close_rel(got, want, rel, abs_=0.0):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    bound = rel * np.abs(want) + abs_
    bad = err > bound
    assert not bad.any(), (f"{bad.sum()} of {bad.size} elements out of tolerance; worst "
                           f"err {err.max():.3e} at want {want.flat[err.argmax()]:.6e}")


def assert_bf16_close(got_bits, want_bits, rel=1e-2):
    got = obf16.decode(got_bits)
    want = obf16.decode(want_bits)
    rms = float(np.sqrt(np.mean(want ** 2)))
    bound = rel * np.maximum(np.abs(want), rms)
    err = np.abs(got - want)
    assert (err <= bound).all(), f"worst err {err.max():.3e} vs bound {bound.flat[err.argmax()]:.3e}"
    fro = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert fro <= rel, f"Frobenius error {fro:.3e}"


def run_job_to_completion(job, max_resumes=100000):
    """Drive a job through wait/resume cycles; returns the list of states seen."""
    import paper_2410_07381_amd.binding as B
    states = []
    for _ in range(max_resumes):
        st = job.wait()
        states.append(st)
        if st == B.JOB_COMPLETE:
            return states
        job.resume()
    raise AssertionError("job did not complete")


def oracle_block_sums(x_host, blocks=None):
    """Per-block partial sums of the reduction kernel from the oracle, for all logical
    blocks or for the listed ones.  Returns (block indices, partials)."""
    n = int(x_host.size)
    nb = OK.grid_of("reduce_sum", {"n": n})[0]
    idx = np.arange(nb) if blocks is None else np.asarray(sorted(set(int(b) for b in blocks)))
    a = {"x": x_host.reshape(-1), "n": n, "partial": np.zeros(nb, np.float32)}
    for b in idx:
        OK.exec_block("reduce_sum", (int(b), 0, 0), (nb, 1, 1), a)
    return idx, a["partial"][idx]


def oracle_softmax_rows(x_rows):
    """Row softmax of a [rows, cols] fp32 array through the oracle's logical blocks."""
    rows, cols = x_rows.shape
    a = {"x": np.ascontiguousarray(x_rows), "y": np.zeros((rows, cols), np.float32), "rows": rows,
         "cols": cols}
    OS.run_native("softmax_f32", OK.grid_of("softmax_f32", a), a)
    return a["y"]
