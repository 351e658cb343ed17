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
def _explore(make, max_preempts):
    """Walk EVERY interleaving of worker micro-steps and EVERY moment at which the flag
    may be raised (up to max_preempts times) of the machine `make()` builds.  Returns a
    dict of findings."""
    found = {"lost": False, "dup": False, "prefix_broken": False, "finals": 0, "max_depth": 0}
    seen = set()
    m0 = make()
    total = m0.total

    def rec(m, counts, used, depth):
        k = (m.key(), counts, used)
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

    rec(m0, (0,) * total, 0, 0)
    found["states"] = len(seen)
    return found


def _paper(total, workers, order="check_then_fetch", chunk=1):
    return lambda: S.PtbMachine(total, workers, order=order, chunk=chunk)


def _folded(total, workers, chunk=1, **kw):
    return lambda: S.FoldedPtbMachine(total, workers, chunk=chunk, **kw)


@pytest.mark.parametrize("total,workers", [(1, 1), (2, 3), (4, 2), (5, 3), (6, 2), (6, 3)])
def test_exactly_once_under_every_interleaving_and_preemption_point(total, workers):
    for make in (_paper(total, workers), _folded(total, workers),
                 _folded(total, workers, single_pass=False),
                 _folded(total, workers, word0=(1 << 32) - 2)):     # the word wraps mid-run
        f = _explore(make, max_preempts=2)
        assert f["finals"] > 0
        assert not f["lost"] and not f["dup"] and not f["prefix_broken"]


@pytest.mark.parametrize("total,workers,chunk", [(5, 2, 2), (6, 3, 2), (7, 2, 3), (3, 2, 4)])
def test_exactly_once_with_chunked_fetch(total, workers, chunk):
    # taking several consecutive task indices per fetch keeps exactly-once and the prefix
    # property as long as every fetched index is run before the worker leaves
    for make in (_paper(total, workers, chunk=chunk), _folded(total, workers, chunk=chunk),
                 _folded(total, workers, chunk=chunk, single_pass=False),
                 _folded(total, workers, chunk=chunk, word0=(1 << 32) - 3)):
        f = _explore(make, max_preempts=2)
        assert f["finals"] > 0
        assert not f["lost"] and not f["dup"] and not f["prefix_broken"]


def test_chunked_fetch_drains_on_a_chunk_boundary():
    cov, log = S.run_ptb(None, (37, 1, 1), {}, 3, preempt_points=[5, 18], seed=2, chunk=4)
    assert cov.exactly_once()
    assert log == [8, 20, 37]
    assert (cov.segment[:8] == 0).all() and (cov.segment[8:20] == 1).all()
    assert (cov.segment[20:] == 2).all()


def test_brute_force_detects_the_wrong_order():
    f = _explore(_paper(4, 2, order="fetch_then_check"), max_preempts=1)
    assert f["lost"], "fetch-before-check must lose a block on some interleaving"
    assert f["prefix_broken"]


def test_brute_force_detects_wrong_one_word_forms():
    # resuming without moving the base: the fetches that failed after the request have
    # advanced the word, so indices are skipped
    f = _explore(_folded(4, 2, variant="stale_base"), max_preempts=1)
    assert f["lost"]
    # reading the progress off the word after a request counts those failed fetches as work
    f = _explore(_folded(4, 2, variant="counter_progress"), max_preempts=1)
    assert f["prefix_broken"] or f["lost"]


@pytest.mark.parametrize("total,workers,chunk", [(5, 2, 1), (6, 3, 2), (7, 2, 3), (4, 3, 1)])
def test_one_word_machine_is_the_papers_machine_step_for_step(total, workers, chunk):
    """Driven by the same sequence of worker steps and flag raises, the one-word machine
    and the paper's counter-plus-flag machine run the same blocks in the same segments and
    report the same progress at every drain (every schedule, by exhaustive walk)."""
    seen = set()

    def rec(a, b, used, depth):
        k = (a.key(), b.key(), used)
        if k in seen:
            return
        seen.add(k)
        assert depth < 200
        assert a.live() == b.live() and a.flag == b.flag
        live = a.live()
        if not live:
            assert a.progress() == b.progress()
            a2, b2 = a.clone(), b.clone()
            ra, rb = a2.resume(), b2.resume()
            assert ra == rb and a2.progress_log == b2.progress_log
            if ra:
                rec(a2, b2, used, depth + 1)
            return
        if not a.flag and used < 2:
            a2, b2 = a.clone(), b.clone()
            a2.raise_flag()
            b2.raise_flag()
            rec(a2, b2, used + 1, depth + 1)
        for w in live:
            xa, xb = [], []
            a2 = a.clone(on_exec=lambda i, s_, ww: xa.append((i, s_, ww)))
            b2 = b.clone(on_exec=lambda i, s_, ww: xb.append((i, s_, ww)))
            a2.step(w)
            b2.step(w)
            assert xa == xb
            rec(a2, b2, used, depth + 1)

    # (without the single-pass shortcut the two machines have the same states throughout)
    rec(S.PtbMachine(total, workers, chunk=chunk),
        S.FoldedPtbMachine(total, workers, chunk=chunk, single_pass=False, word0=(1 << 32) - 1),
        0, 0)
    assert len(seen) > 50


def test_single_pass_leaves_without_a_second_fetch():
    m = S.FoldedPtbMachine(8, 4, chunk=2)              # 4 workers x 2 cover all 8 blocks
    assert m.single
    ran = []
    m.on_exec = lambda i, s_, w: ran.append(i)
    for w in range(4):
        m.step(w)                                      # one fetch each
    for _ in range(2):
        for w in range(4):
            m.step(w)
    assert m.drained() and sorted(ran) == list(range(8))
    assert (m.word - m.base) % S.WORD == 8             # no failing fetch was made
    m = S.FoldedPtbMachine(9, 4, chunk=2)              # one block too many for a single pass
    assert not m.single


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


# ---- invariants over random grids, worker counts, chunks, preemption points and seeds ---------
from hypothesis import given, settings, strategies as st  # noqa: E402


@settings(max_examples=60, deadline=None)
@given(gx=st.integers(1, 9), gy=st.integers(1, 5), gz=st.integers(1, 3), workers=st.integers(1, 12),
       chunk=st.integers(1, 5), seed=st.integers(0, 1000), word0=st.sampled_from([0, 7, (1 << 32) - 3, 1 << 31]),
       raw_pts=st.lists(st.integers(0, 200), max_size=4), machine=st.sampled_from(["folded", "paper"]))
def test_ptb_invariants_hold_for_any_run(gx, gy, gz, workers, chunk, seed, word0, raw_pts, machine):
    """Whatever the grid, the worker count, the chunk, the moments of the requests, the
    interleaving and the value the shared word starts from (near its wrap-around included):
    every block runs exactly once with the coordinates of its index, the progress values are
    non-decreasing, each is a request point rounded up to what the chunks allow and never beyond
    the grid, and a block's segment is the one whose [start, stop) range holds its index."""
    grid = (gx, gy, gz)
    total = G.total_blocks(grid)
    pts = sorted(p % (total + 1) for p in raw_pts)
    kw = {"word0": word0} if machine == "folded" else {}
    cov, log = S.run_ptb(None, grid, {}, workers, preempt_points=pts, seed=seed, chunk=chunk,
                         machine=machine, **kw)
    assert cov.exactly_once()
    assert log[-1] == total and all(a <= b for a, b in zip(log, log[1:]))
    assert all(0 <= p <= total for p in log)
    edges = [0] + log
    for s in range(len(edges) - 1):
        assert (cov.segment[edges[s]:edges[s + 1]] == s).all()
    for idx in range(total):
        assert tuple(int(v) for v in cov.bidx[idx]) == G.delinearize(idx, grid)
    if chunk == 1:
        assert log[:-1] == [p for p in pts if p < total] or log[:-1] == pts[:len(log) - 1]


@settings(max_examples=60, deadline=None)
@given(total=st.integers(1, 300), slice_blocks=st.integers(1, 64),
       stops=st.lists(st.integers(1, 40), max_size=3, unique=True))
def test_sliced_invariants_hold_for_any_run(total, slice_blocks, stops):
    """Slices cover [0, total) in order, each block once, the last slice is the remainder, and
    a stop after n slices starts a new segment at offset n * slice_blocks."""
    cov, resumes = S.run_sliced(None, (total, 1, 1), {}, slice_blocks, preempt_after_slices=sorted(stops))
    assert cov.exactly_once()
    nslices = -(-total // slice_blocks)
    seg, want_resumes = 0, []
    for sl in range(nslices):
        lo, hi = sl * slice_blocks, min((sl + 1) * slice_blocks, total)
        assert (cov.segment[lo:hi] == seg).all()
        if (sl + 1) in stops and sl + 1 < nslices:
            seg += 1
            want_resumes.append(hi)
    assert resumes == want_resumes
