"""Profile-guided choice of a launch configuration, and the scheduler's decision rule.

Section 4.2: for each best-effort kernel the scheduler builds candidate
configurations of both kinds (persistent-worker counts that are multiples of the
number of compute units and fit the occupancy limit; slice sizes covering
different fractions of the grid), measures each, estimates its turnaround latency,
and keeps the best-performing one whose estimate respects the threshold.

Turnaround estimate: for a sliced kernel it is the measured time of one slice; for
a persistent-worker kernel it is Eq. 1,
    turnaround = kernel_latency * worker_blocks / total_blocks,
i.e. the whole-kernel time divided by the number of blocks each worker handles.

Readings where the paper is silent: if no candidate meets the threshold the one
with the smallest estimate is taken; ties go to the persistent-worker form, then to
fewer workers / larger slices.
"""
from __future__ import annotations

DEFAULT_THRESHOLD_MS = 0.0316
DEFAULT_PROFILE_RUNS = 10


def ptb_turnaround_ms(kernel_latency_ms, worker_blocks, total_blocks):
    """Eq. 1."""
    return kernel_latency_ms * worker_blocks / total_blocks


def sliced_turnaround_ms(slice_latency_ms, in_flight=1, n_slices=None):
    """Section 4.2: the completion time of a single slice.  Where more than one slice is
    kept enqueued (`in_flight`; the paper enqueues one), none of them can be recalled, so
    the estimate is the completion time of all of them; a kernel never has more slices in
    flight than it has slices."""
    if in_flight < 1:
        raise ValueError("in_flight must be positive")
    q = in_flight if n_slices is None else min(in_flight, n_slices)
    return slice_latency_ms * q


def ptb_candidates(total_blocks, num_cus, max_blocks_per_cu):
    """Worker counts k * num_cus for k = 1 .. occupancy limit, capped at the grid size."""
    out = []
    for k in range(1, max_blocks_per_cu + 1):
        w = min(k * num_cus, total_blocks)
        if w not in out:
            out.append(w)
    return out


def slice_candidates(total_blocks, fractions=(1, 1 / 2, 1 / 4, 1 / 8, 1 / 16, 1 / 32, 1 / 64,
                                             1 / 128, 1 / 256)):
    """Blocks per slice for slices of the given shares of the grid (Section 4.2 names no
    shares; the whole grid is one of them: one launch, which is all a kernel shorter than
    the threshold needs)."""
    out = []
    for f in fractions:
        n = max(1, int(total_blocks * f))
        if n not in out:
            out.append(n)
    return out


def select_config(measurements, threshold_ms=DEFAULT_THRESHOLD_MS):
    """`measurements`: list of dicts {kind: 'ptb'|'sliced', param, latency_ms,
    turnaround_ms}.  Returns the chosen dict."""
    if not measurements:
        raise ValueError("no candidates")

    def tie(m):  # persistent-worker before sliced; fewer workers; larger slices
        return (0, m["param"]) if m["kind"] == "ptb" else (1, -m["param"])

    ok = [m for m in measurements if m["turnaround_ms"] <= threshold_ms]
    if ok:
        return min(ok, key=lambda m: (m["latency_ms"],) + tie(m))
    return min(measurements, key=lambda m: (m["turnaround_ms"],) + tie(m))


class ProfileCache:
    """Measurements keyed by (kernel, grid, block); one candidate is profiled per real
    invocation of the kernel, and the configuration is fixed once all are measured."""

    def __init__(self, threshold_ms=DEFAULT_THRESHOLD_MS):
        self.threshold_ms = threshold_ms
        self.meas = {}
        self.chosen = {}

    def lookup(self, key):
        return self.chosen.get(key)

    def next_unmeasured(self, key, candidates):
        done = self.meas.get(key, {})
        for c in candidates:
            if c not in done:
                return c
        return None

    def record(self, key, cand, latency_ms, total_blocks, slice_latency_ms=None):
        """cand = (kind, param) or (kind, param, n): n task indices per fetch for persistent
        workers (each worker then holds n blocks, so Eq. 1 is taken with n times the worker
        blocks), n slices kept enqueued for a sliced candidate.  The time of one slice
        defaults to the kernel's time divided by its number of slices."""
        kind, param = cand[0], cand[1]
        n = cand[2] if len(cand) > 2 else 1
        if kind == "ptb":
            t = ptb_turnaround_ms(latency_ms, param * n, total_blocks)
        else:
            slices = -(-total_blocks // param)
            if slice_latency_ms is None:
                slice_latency_ms = latency_ms / slices
            t = sliced_turnaround_ms(slice_latency_ms, n, n_slices=slices)
        self.meas.setdefault(key, {})[cand] = {
            "kind": kind, "param": param, "latency_ms": latency_ms, "turnaround_ms": t}

    def finalize(self, key, candidates):
        if self.next_unmeasured(key, candidates) is not None:
            return None
        self.chosen[key] = select_config([self.meas[key][c] for c in candidates],
                                         self.threshold_ms)
        return self.chosen[key]


def scheduler_action(hi_has_new_kernel, hi_running, be_state):
    """One pass of the priority-aware loop (Section 4.2) for one high-priority and one
    best-effort client.  be_state in {'none', 'running', 'stopped', 'pending'}.
    Returns the ordered list of actions taken in this pass."""
    acts = []
    if hi_has_new_kernel:
        acts += ["preempt_best_effort", "launch_hi"]
        hi_running = True
    if hi_running:
        return acts                       # best-effort clients are not visited
    if be_state == "pending":
        acts.append("launch_be")
    elif be_state == "stopped":
        acts.append("resume_be")
    return acts
