"""Logical grid arithmetic.

A kernel is a grid of independent thread blocks that may run in any order
(Background, "GPU architecture and programming model").  Both transformations
rebuild the original block index from one integer: slicing adds a block offset to
the sub-kernel's own block index (Section 4.1, slicing transformation); the
persistent-worker form maps a fetched task index to the block index "by referring
to the original kernel's grid dimension" (Section 4.1, preemption transformation).
The paper does not fix the order for multi-dimensional grids; x varies fastest
here.
"""


def total_blocks(grid):
    gx, gy, gz = grid
    return int(gx) * int(gy) * int(gz)


def delinearize(idx, grid):
    gx, gy, _ = grid
    bx = idx % gx
    by = (idx // gx) % gy
    bz = idx // (gx * gy)
    return (bx, by, bz)


def linearize(b, grid):
    gx, gy, _ = grid
    return b[0] + gx * (b[1] + gy * b[2])
