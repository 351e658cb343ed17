"""Pins for the turnaround estimate (Eq. 1), the candidate sets, the selection rule and
the scheduler's per-pass decision."""
import json
import os

import pytest

from oracle import profiler as P


def test_eq1_cases_from_fixture(golden_dir):
    with open(os.path.join(golden_dir, "turnaround.json")) as f:
        g = json.load(f)
    assert P.DEFAULT_THRESHOLD_MS == g["threshold_ms"]
    assert P.DEFAULT_PROFILE_RUNS == g["profile_runs"]
    for c in g["cases"]:
        got = P.ptb_turnaround_ms(c["kernel_latency_ms"], c["worker_blocks"], c["total_blocks"])
        assert got == pytest.approx(c["turnaround_ms"], rel=1e-12)


def test_eq1_limits():
    # as many workers as blocks: every worker runs one block, nothing to gain
    assert P.ptb_turnaround_ms(3.0, 64, 64) == 3.0
    # one worker: the estimate is the per-block time
    assert P.ptb_turnaround_ms(3.0, 1, 64) == pytest.approx(3.0 / 64)
    # linear in the worker count
    assert P.ptb_turnaround_ms(1.0, 512, 4096) == 2 * P.ptb_turnaround_ms(1.0, 256, 4096)


def test_sliced_turnaround_hand_table():
    # one slice at a time (the paper's form): the time of one slice
    assert P.sliced_turnaround_ms(0.010) == 0.010
    # three slices of 10 us kept enqueued: all three must finish, 30 us
    assert P.sliced_turnaround_ms(0.010, 3) == pytest.approx(0.030)
    # a kernel of two slices cannot have three in flight
    assert P.sliced_turnaround_ms(0.010, 3, n_slices=2) == pytest.approx(0.020)
    assert P.sliced_turnaround_ms(0.010, 8, n_slices=1) == pytest.approx(0.010)
    with pytest.raises(ValueError):
        P.sliced_turnaround_ms(0.010, 0)


@pytest.mark.parametrize("d,q,n", [(4, 1, 6), (3, 2, 7), (5, 3, 4), (2, 4, 3), (1, 2, 9)])
def test_sliced_turnaround_is_the_worst_drain_of_a_simulated_queue(d, q, n):
    """A queue simulated tick by tick: n slices of d ticks each run one after another, the
    driver keeps at most q enqueued and stops enqueueing when the request arrives.  The
    longest wait, over every arrival tick, for the enqueued slices to finish is what the
    estimate must equal."""
    worst = 0
    for t_req in range(n * d + 1):
        issued = finished = busy_left = t = 0
        while True:
            # within a tick: the driver tops the queue up, then (at t_req) the request arrives
            if t <= t_req:
                while issued < n and issued - finished < q:
                    issued += 1
            if busy_left == 0 and issued > finished:
                busy_left = d                    # the next enqueued slice starts
            if t >= t_req and issued == finished:
                break                            # nothing enqueued is left: drained
            if busy_left > 0:
                busy_left -= 1
                if busy_left == 0:
                    finished += 1
            t += 1
        worst = max(worst, t - t_req)
    assert worst == P.sliced_turnaround_ms(d, q, n_slices=n)


def test_candidates():
    assert P.ptb_candidates(65536, 256, 4) == [256, 512, 768, 1024]
    assert P.ptb_candidates(256, 256, 8) == [256]            # capped at the grid size
    assert P.ptb_candidates(600, 256, 3) == [256, 512, 600]
    assert P.slice_candidates(65536)[:4] == [65536, 32768, 16384, 8192]
    assert P.slice_candidates(4) == [4, 2, 1]


def _m(kind, param, lat, turn):
    return {"kind": kind, "param": param, "latency_ms": lat, "turnaround_ms": turn}


def test_selection_rule():
    t = 0.0316
    ms = [_m("ptb", 256, 1.30, 0.005), _m("ptb", 512, 1.10, 0.010), _m("ptb", 2048, 1.00, 0.040),
          _m("sliced", 4096, 1.05, 0.066), _m("sliced", 512, 1.20, 0.009)]
    assert P.select_config(ms, t)["param"] == 512 and P.select_config(ms, t)["kind"] == "ptb"
    # loosen the bound: the fastest overall wins
    assert P.select_config(ms, 1.0)["param"] == 2048
    # nothing complies: smallest turnaround
    assert P.select_config(ms, 0.001)["param"] == 256
    # tie on latency: persistent-worker form first, then fewer workers
    tie = [_m("sliced", 64, 1.0, 0.01), _m("ptb", 512, 1.0, 0.01), _m("ptb", 256, 1.0, 0.01)]
    assert P.select_config(tie, t) == tie[2]
    with pytest.raises(ValueError):
        P.select_config([], t)


def test_profile_cache_one_candidate_per_invocation():
    cache = P.ProfileCache()
    key = ("reduce_sum", (65536, 1, 1), (256, 1, 1))
    cands = [("ptb", 256), ("ptb", 512), ("sliced", 4096)]
    assert cache.lookup(key) is None
    lat = {("ptb", 256): 1.2, ("ptb", 512): 1.0, ("sliced", 4096): 0.9}
    for i in range(3):
        c = cache.next_unmeasured(key, cands)
        assert c == cands[i]
        assert cache.finalize(key, cands) is None
        cache.record(key, c, lat[c], 65536, slice_latency_ms=0.9 / 16)
    assert cache.next_unmeasured(key, cands) is None
    chosen = cache.finalize(key, cands)
    # sliced(4096): turnaround 0.056 ms > 0.0316; ptb(512): 1.0*512/65536 = 0.0078 ms
    assert (chosen["kind"], chosen["param"]) == ("ptb", 512)
    assert cache.lookup(key) is chosen


def test_scheduler_pass():
    A = P.scheduler_action
    assert A(True, False, "running") == ["preempt_best_effort", "launch_hi"]
    assert A(False, True, "stopped") == []                   # hi-pri in flight: no resume
    assert A(False, False, "stopped") == ["resume_be"]
    assert A(False, False, "pending") == ["launch_be"]
    assert A(False, False, "running") == []
    assert A(True, True, "pending") == ["preempt_best_effort", "launch_hi"]
