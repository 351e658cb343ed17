"""Launch schedules on the CPU: native, sliced, persistent-worker with preemption.

Each schedule decides WHICH logical block runs in WHICH launch segment; the block
body itself comes from `kernels.exec_block`.  A per-block coverage record is kept
so that "every logical block ran exactly once" can be checked directly.

Slicing (Section 4.1, slicing transformation): a sub-kernel covers blocks
[offset, offset+n) and rebuilds the original block index as offset + blockIdx;
sub-kernels are issued one at a time (Section 4.2).  Re-launching the original
kernel on a smaller grid WITHOUT the offset is the wrong scheme the paper warns
about; it is kept here as a negative control.

Persistent workers (Section 4.1, preemption transformation): W worker blocks loop;
at the start of an iteration a worker checks the preemption flag, then fetches and
increments the global task counter, maps the task index to the original block
index, runs that block, synchronises, and repeats.  Progress lives entirely in the
counter, so a drained kernel is resumed by launching the workers again without
resetting it.
"""
from __future__ import annotations

import numpy as np

from . import grid as G
from . import kernels as K


class Coverage:
    """Per-logical-block record: execution count, rebuilt block index, launch segment."""

    def __init__(self, grid):
        n = G.total_blocks(grid)
        self.grid = tuple(int(g) for g in grid)
        self.count = np.zeros(n, dtype=np.uint32)
        self.bidx = np.full((n, 3), 0xFFFFFFFF, dtype=np.uint32)
        self.segment = np.full(n, 0xFFFFFFFF, dtype=np.uint32)

    def mark(self, slot, b, segment):
        self.count[slot] += 1
        self.bidx[slot] = b
        self.segment[slot] = segment

    def exactly_once(self):
        return bool((self.count == 1).all())


def _run_block(name, idx, grid, args, cov, segment):
    b = G.delinearize(idx, grid)
    if name is not None:
        K.exec_block(name, b, grid, args)
    cov.mark(G.linearize(b, grid), b, segment)


def run_native(name, grid, args):
    cov = Coverage(grid)
    for idx in range(G.total_blocks(grid)):
        _run_block(name, idx, grid, args, cov, 0)
    return cov


def slice_offsets(total, slice_blocks):
    """Offsets of the sub-kernels; the last one takes the remainder."""
    if slice_blocks <= 0:
        raise ValueError("slice_blocks must be positive")
    return list(range(0, total, slice_blocks))


def run_sliced(name, grid, args, slice_blocks, preempt_after_slices=()):
    """Issue sub-kernels one at a time.  `preempt_after_slices` holds slice counts
    after which the high-priority job intervened; the saved offset is the resume
    point and a new segment starts there.  Returns (coverage, resume offsets)."""
    total = G.total_blocks(grid)
    cov = Coverage(grid)
    stops = set(int(s) for s in preempt_after_slices)
    segment, issued, resumes = 0, 0, []
    for off in slice_offsets(total, slice_blocks):
        n = min(slice_blocks, total - off)
        for j in range(n):                      # sub-kernel block j -> logical off + j
            _run_block(name, off + j, grid, args, cov, segment)
        issued += 1
        if issued in stops and off + n < total:
            segment += 1
            resumes.append(off + n)
    return cov, resumes


def run_naive_sliced(name, grid, args, slice_blocks):
    """Negative control: the original kernel launched once per slice on a
    slice-sized grid with no offset, so every launch sees block indices 0..n-1."""
    total = G.total_blocks(grid)
    cov = Coverage(grid)
    for off in slice_offsets(total, slice_blocks):
        n = min(slice_blocks, total - off)
        for j in range(n):
            _run_block(name, j, grid, args, cov, 0)
    return cov


# --------------------------------------------------------------------- persistent workers
CHECK, FETCHED, EXITED = 0, 1, 2


class PtbMachine:
    """Micro-step model of W persistent workers sharing one counter and one flag.

    A worker is in CHECK (about to start an iteration), FETCHED(idx) (holds task
    indices it has not run yet) or EXITED.  `step(w)` advances worker w by one
    micro-step.  `order` = "check_then_fetch" is the paper's order ("at the start of
    each iteration, workers check this flag").  "fetch_then_check" is a deliberately
    wrong variant (a fetched index is dropped when the flag is seen) kept so the
    tests can show the brute-force checker is not vacuous.
    """

    def __init__(self, total, workers, order="check_then_fetch", on_exec=None, chunk=1):
        self.total = int(total)
        self.W = int(workers)
        self.order = order
        # consecutive task indices taken per fetch (1 is the paper's form)
        self.chunk = int(chunk)
        if self.chunk < 1:
            raise ValueError("chunk must be positive")
        self.held_end = [-1] * self.W
        self.counter = 0
        self.flag = False
        self.state = [CHECK] * self.W
        self.held = [-1] * self.W
        self.segment = 0
        self.on_exec = on_exec
        self.progress_log = []

    # -- copying (for exhaustive search) ------------------------------------------------
    def clone(self, on_exec=None):
        m = PtbMachine.__new__(PtbMachine)
        m.total, m.W, m.order = self.total, self.W, self.order
        m.chunk, m.held_end = self.chunk, list(self.held_end)
        m.counter, m.flag, m.segment = self.counter, self.flag, self.segment
        m.state, m.held = list(self.state), list(self.held)
        m.on_exec = on_exec
        m.progress_log = list(self.progress_log)
        return m

    def key(self):
        """Everything the future of the machine depends on (for exhaustive search)."""
        return (self.counter, self.flag, tuple(self.state), tuple(self.held), tuple(self.held_end),
                self.segment)

    # -- queries ------------------------------------------------------------------------
    def live(self):
        return [w for w in range(self.W) if self.state[w] != EXITED]

    def drained(self):
        return all(s == EXITED for s in self.state)

    def progress(self):
        return min(self.counter, self.total)

    def complete(self):
        return self.drained() and self.progress() == self.total

    # -- transitions --------------------------------------------------------------------
    def raise_flag(self):
        self.flag = True

    def step(self, w):
        s = self.state[w]
        if s == EXITED:
            raise RuntimeError("stepping an exited worker")
        if s == CHECK:
            if self.order == "check_then_fetch":
                if self.flag:
                    self.state[w] = EXITED
                    return
                idx = self.counter
                n = self.chunk
                self.counter += n
                if idx >= self.total:
                    self.state[w] = EXITED
                    return
                self.state[w], self.held[w] = FETCHED, idx
                self.held_end[w] = min(idx + n, self.total)
            else:  # wrong order: fetch first, then honour the flag and drop the index
                idx = self.counter
                n = self.chunk
                self.counter += n
                if idx >= self.total or self.flag:
                    self.state[w] = EXITED
                    return
                self.state[w], self.held[w] = FETCHED, idx
                self.held_end[w] = min(idx + n, self.total)
        else:  # FETCHED: run one held block, reach the barrier; loop when none is left
            idx = self.held[w]
            if self.on_exec is not None:
                self.on_exec(idx, self.segment, w)
            if idx + 1 < self.held_end[w]:
                self.held[w] = idx + 1   # a fetched index is always run before the flag counts
            else:
                self.state[w], self.held[w], self.held_end[w] = CHECK, -1, -1

    def resume(self):
        """Relaunch after a drain: flag cleared, counter kept."""
        if not self.drained():
            raise RuntimeError("resume before drain")
        self.progress_log.append(self.progress())
        if self.progress() >= self.total:
            return False
        self.flag = False
        self.segment += 1
        self.state = [CHECK] * self.W
        self.held = [-1] * self.W
        self.held_end = [-1] * self.W
        return True


WORD = 1 << 32            # the shared word is 32 bits wide and wraps
PREEMPT_STEP = 1 << 31    # what a preemption request adds to it


class FoldedPtbMachine(PtbMachine):
    """The same worker loop with the flag folded into the counter: ONE shared 32-bit word.

    The paper keeps two variables, a task counter and a boolean flag, and a worker reads the
    flag, then fetches and increments the counter.  Here a worker does one fetch-and-add on
    one word and compares what it got with the end of the grid; a preemption request is
    itself a fetch-and-add, of 2^31, on that word, after which every fetch returns an index
    beyond any grid and the worker leaves exactly as it would on seeing the flag.  What the
    request's own fetch-and-add returned is the number of indices handed out before it:
    the progress.  Fetches that fail after the request still add to the word, so the word no
    longer shows the progress; instead of resetting it, the host moves its `base` (the value
    of the word that stands for task index 0) so that the next index handed out is again
    `progress`.  The word is never reset and wraps modulo 2^32; indices are differences
    modulo 2^32, so the grid must be smaller than 2^31 blocks.

    `single_pass`: when the workers' first fetches alone cover every index left
    (chunk x workers >= blocks left at the start of the segment), a worker that has run what
    it fetched leaves without a second, necessarily failing, fetch.

    `variant` selects deliberately wrong forms, kept as negative controls for the
    exhaustive checker: "stale_base" resumes without moving the base, "counter_progress"
    reads the progress off the word after a request.
    """

    def __init__(self, total, workers, on_exec=None, chunk=1, word0=0, variant="right",
                 single_pass=True):
        super().__init__(total, workers, on_exec=on_exec, chunk=chunk)
        if self.total >= PREEMPT_STEP:
            raise ValueError("grid too large for a 32-bit word with a folded request")
        self.word = int(word0) % WORD
        self.base = self.word
        self.variant = variant
        self.allow_single = bool(single_pass)
        self.flag_progress = None
        self._open_segment(0)

    def _open_segment(self, start):
        self.seg_start = start
        self.single = self.allow_single and self.chunk * self.W >= self.total - start

    def clone(self, on_exec=None):
        m = FoldedPtbMachine.__new__(FoldedPtbMachine)
        m.__dict__.update(self.__dict__)
        m.held_end, m.state, m.held = list(self.held_end), list(self.state), list(self.held)
        m.progress_log = list(self.progress_log)
        m.on_exec = on_exec
        return m

    def key(self):
        return (self.word, self.base, self.flag, self.flag_progress, tuple(self.state),
                tuple(self.held), tuple(self.held_end), self.segment, self.single)

    @property
    def counter(self):
        """Task indices handed out, as the paper's counter would show them (for callers
        that watch the counter to decide when to raise the request)."""
        if self.flag:
            return self.flag_progress_raw
        return (self.word - self.base) % WORD

    @counter.setter
    def counter(self, v):      # the base class initialises the attribute; the word is the state
        pass

    def progress(self):
        if self.flag and self.variant != "counter_progress":
            return self.flag_progress
        return min((self.word - self.base) % WORD, self.total)

    def raise_flag(self):
        if self.flag:
            return
        old = self.word
        self.word = (self.word + PREEMPT_STEP) % WORD
        self.flag = True
        self.flag_progress_raw = (old - self.base) % WORD
        self.flag_progress = min(self.flag_progress_raw, self.total)

    def step(self, w):
        s = self.state[w]
        if s == EXITED:
            raise RuntimeError("stepping an exited worker")
        if s == CHECK:
            old = self.word
            self.word = (self.word + self.chunk) % WORD
            idx = (old - self.base) % WORD
            if idx >= self.total:              # grid exhausted, or a request folded in
                self.state[w] = EXITED
                return
            self.state[w], self.held[w] = FETCHED, idx
            self.held_end[w] = min(idx + self.chunk, self.total)
        else:
            idx = self.held[w]
            if self.on_exec is not None:
                self.on_exec(idx, self.segment, w)
            if idx + 1 < self.held_end[w]:
                self.held[w] = idx + 1
            elif self.single:
                self.state[w], self.held[w], self.held_end[w] = EXITED, -1, -1
            else:
                self.state[w], self.held[w], self.held_end[w] = CHECK, -1, -1

    def resume(self):
        if not self.drained():
            raise RuntimeError("resume before drain")
        p = self.progress()
        self.progress_log.append(p)
        if p >= self.total:
            return False
        if self.variant != "stale_base":
            self.base = (self.word - p) % WORD   # the next index handed out is p again
        self.flag = False
        self.flag_progress = None
        self.segment += 1
        self.state = [CHECK] * self.W
        self.held = [-1] * self.W
        self.held_end = [-1] * self.W
        self._open_segment(p)
        return True


def run_ptb(name, grid, args, workers, preempt_points=(), seed=0, chunk=1, machine="folded",
            word0=0):
    """Run a kernel as `workers` persistent workers under a seeded random
    interleaving, on the one-word machine the GPU path uses (machine="folded") or on the
    paper's two-variable one (machine="paper"); both give the same coverage and progress.
    The flag is raised when the counter first reaches (or, with chunk > 1, first passes)
    each value in `preempt_points` (ascending); after every drain the kernel is resumed.
    Returns (coverage, progress value observed at each drain)."""
    total = G.total_blocks(grid)
    cov = Coverage(grid)

    def on_exec(idx, segment, w):
        _run_block(name, idx, grid, args, cov, segment)

    if machine == "folded":
        m = FoldedPtbMachine(total, workers, on_exec=on_exec, chunk=chunk, word0=word0)
    else:
        m = PtbMachine(total, workers, on_exec=on_exec, chunk=chunk)
    rng = np.random.Generator(np.random.PCG64(seed))
    pts = sorted(int(p) for p in preempt_points)
    nxt = 0
    while True:
        if not m.flag and nxt < len(pts) and pts[nxt] <= m.counter:
            m.raise_flag()
            nxt += 1
            while nxt < len(pts) and pts[nxt] < m.counter:
                nxt += 1                 # points already passed are part of the same drain
        live = m.live()
        if live:
            m.step(live[int(rng.integers(len(live)))])
            continue
        if not m.resume():
            break
    return cov, m.progress_log
