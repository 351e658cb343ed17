"""Pins for the oracle's schedule simulators: the paper's worked examples, brute force
over every interleaving on tiny grids, and a negative control showing the checker
would catch the wrong flag/fetch order."""
import json
import os

import numpy as np
import pytest

from oracle import grid as G
from oracle import schedules as S


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


# ------------------------------------------------------------------ paper's worked examples
def test_slicing_example_from_paper(golden_dir):
    g = _load(golden_dir, "slicing_example.json")
    total, n = g["total_blocks"], g["slice_blocks"]
    assert S.slice_offsets(total, n) == g["offsets"]
    cov, resumes = S.run_sliced(None, (total, 1, 1), {}, n)
    assert cov.exactly_once() and resumes == []
    # sub-kernel 2 (1-indexed) = offset 4, blocks 4..7
    off = g["offsets"][1]
    assert [off + j for j in range(n)] == g["sub_kernel_2_blocks"]
    assert [int(b) for b in cov.bidx[4:8, 0]] == g["sub_kernel_2_blocks"]


def test_naive_relaunch_is_wrong(golden_dir):
    g = _load(golden_dir, "slicing_example.json")
    cov = S.run_naive_sliced(None, (g["total_blocks"], 1, 1), {}, g["slice_blocks"])
    assert cov.count.tolist() == g["naive_counts"]
    assert not cov.exactly_once()


def test_ptb_example_from_paper(golden_dir):
    g = _load(golden_dir, "ptb_example.json")
    grid = (g["total_blocks"], 1, 1)
    assert list(G.delinearize(g["task_index"], grid)) == g["block_index"]
    for seed in range(20):
        cov, log = S.run_ptb(None, grid, {}, g["workers"], seed=seed)
        assert cov.exactly_once()
        assert log == [g["total_blocks"]]
        assert (cov.bidx[:, 0] == np.arange(16)).all()


# ------------------------------------------------------------------ grid mapping
@pytest.mark.parametrize("grid", [(7, 1, 1), (4, 3, 1), (3, 5, 2), (1, 1, 9), (16, 16, 3)])
def test_delinearize_is_a_bijection_x_fastest(grid):
    total = G.total_blocks(grid)
    seen = set()
    for idx in range(total):
        b = G.delinearize(idx, grid)
        assert all(0 <= b[d] < grid[d] for d in range(3))
        assert G.linearize(b, grid) == idx
        seen.add(b)
    assert len(seen) == total
    if total > 1 and grid[0] > 1:
        assert G.delinearize(1, grid) == (1, 0, 0)          # x varies fastest
    if grid[0] > 0 and grid[1] > 1:
        assert G.delinearize(grid[0], grid) == (0, 1, 0)


def test_slice_remainder_and_resume_offsets():
    cov, resumes = S.run_sliced(None, (10, 1, 1), {}, 4, preempt_after_slices=[1, 2])
    assert cov.exactly_once()
    assert resumes == [4, 8]
    assert cov.segment.tolist() == [0, 0, 0, 0, 1, 1, 1, 1, 2, 2]
    # a preemption after the last slice opens no new segment
    cov, resumes = S.run_sliced(None, (8, 1, 1), {}, 4, preempt_after_slices=[2])
    assert resumes == [] and cov.segment.max() == 0
    with pytest.raises(ValueError):
        S.slice_offsets(8, 0)


# ------------------------------------------------------------------ brute force
def _explore(total, workers, order, max_preempts, chunk=1):
    """Walk EVERY interleaving of worker micro-steps and EVERY moment at which the flag
    may be raised (up to max_preempts times).  Returns a dict of findings."""
    found = {"lost": False, "dup": False, "prefix_broken": False, "finals": 0, "max_depth": 0}
    seen = set()

    def key(m, counts, used):
        return (m.counter, m.flag, tuple(m.state), tuple(m.held), tuple(m.held_end), counts, used,
                m.segment)

    def rec(m, counts, used, depth):
        k = key(m, counts, used)
        if k in seen:
            return
        seen.add(k)
        found["max_depth"] = max(found["max_depth"], depth)
        assert depth < 200, "no termination"
        live = m.live()
        if not live:
            # drained: everything below progress ran exactly once, nothing above ran
            p = m.progress()
            held_back = any(c != 1 for c in counts[:p]) or any(c != 0 for c in counts[p:])
            if held_back:
                found["prefix_broken"] = True
            m2 = m.clone()
            if m2.resume():
                rec(m2, counts, used, depth + 1)
            else:
                found["finals"] += 1
                if any(c == 0 for c in counts):
                    found["lost"] = True
                if any(c > 1 for c in counts):
                    found["dup"] = True
            return
        if not m.flag and used < max_preempts:
            m2 = m.clone()
            m2.raise_flag()
            rec(m2, counts, used + 1, depth + 1)
        for w in live:
            box = []
            m2 = m.clone(on_exec=lambda idx, seg, ww: box.append(idx))
            m2.step(w)
            c2 = counts
            for idx in box:
                c2 = c2[:idx] + (c2[idx] + 1,) + c2[idx + 1:]
            m2.on_exec = None
            rec(m2, c2, used, depth + 1)

    rec(S.PtbMachine(total, workers, order=order, chunk=chunk), (0,) * total, 0, 0)
    found["states"] = len(seen)
    return found


@pytest.mark.parametrize("total,workers", [(1, 1), (2, 3), (4, 2), (5, 3), (6, 2), (6, 3)])
def test_exactly_once_under_every_interleaving_and_preemption_point(total, workers):
    f = _explore(total, workers, "check_then_fetch", max_preempts=2)
    assert f["finals"] > 0
    assert not f["lost"] and not f["dup"] and not f["prefix_broken"]


@pytest.mark.parametrize("total,workers,chunk", [(5, 2, 2), (6, 3, 2), (7, 2, 3), (3, 2, 4)])
def test_exactly_once_with_chunked_fetch(total, workers, chunk):
    # taking several consecutive task indices per fetch keeps exactly-once and the prefix
    # property as long as every fetched index is run before the worker leaves
    f = _explore(total, workers, "check_then_fetch", max_preempts=2, chunk=chunk)
    assert f["finals"] > 0
    assert not f["lost"] and not f["dup"] and not f["prefix_broken"]


def test_chunked_fetch_drains_on_a_chunk_boundary():
    cov, log = S.run_ptb(None, (37, 1, 1), {}, 3, preempt_points=[5, 18], seed=2, chunk=4)
    assert cov.exactly_once()
    assert log == [8, 20, 37]
    assert (cov.segment[:8] == 0).all() and (cov.segment[8:20] == 1).all()
    assert (cov.segment[20:] == 2).all()


def test_brute_force_detects_the_wrong_order():
    f = _explore(4, 2, "fetch_then_check", max_preempts=1)
    assert f["lost"], "fetch-before-check must lose a block on some interleaving"
    assert f["prefix_broken"]


# ------------------------------------------------------------------ seeded runs
@pytest.mark.parametrize("grid,workers,pts", [
    ((64, 1, 1), 8, [5, 17, 40]),
    ((6, 5, 2), 7, [1, 59]),
    ((33, 1, 1), 64, [10]),           # more workers than blocks
    ((16, 1, 1), 4, [0]),             # preempted before the first fetch: empty segment
    ((16, 1, 1), 3, [6, 6, 9]),       # flag seen again before any new fetch: empty segment
])
def test_seeded_ptb_runs(grid, workers, pts):
    total = G.total_blocks(grid)
    for seed in range(5):
        cov, log = S.run_ptb(None, grid, {}, workers, preempt_points=pts, seed=seed)
        assert cov.exactly_once()
        assert log == sorted(pts) + [total]
        # a block belongs to the segment whose [start, stop) range holds its index
        edges = [0] + sorted(pts) + [total]
        for s in range(len(edges) - 1):
            assert (cov.segment[edges[s]:edges[s + 1]] == s).all()
        for idx in range(total):
            assert tuple(int(v) for v in cov.bidx[idx]) == G.delinearize(idx, grid)
