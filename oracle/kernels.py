"""Logical-block bodies of the workload kernels, on the CPU.

Every kernel is defined by (a) its logical grid and (b) what ONE logical block
computes.  Because blocks are independent and order-free (Background, "GPU
architecture and programming model"), the result of the whole kernel is "every
logical block executed exactly once", whatever launch form produced it; the data
result is the textbook operator (y <- a*x + y, sum, A*B, row softmax, LayerNorm,
attention).  Arithmetic is fp64, rounded once to the storage type.

`exec_block(name, b, grid, args)` mutates the output arrays inside `args` exactly
as that block would.  Storage: fp32 arrays are numpy float32; bf16 arrays are
uint16 bit patterns.
"""
from __future__ import annotations

import math

import numpy as np

from . import bf16

THREADS = 256            # threads per logical block, all kernels
REDUCE_PER_THREAD = 16   # elements each thread of a reduce block sums
REDUCE_BLOCK = THREADS * REDUCE_PER_THREAD
GEMM_TILE = 256          # logical output tile edge of the best-effort GEMM
GEMM_SMALL_TILE = 32     # output tile edge of the ragged-edge GEMM (high-priority layer)
GEMM_N128_COLS = 128     # column extent of the 256-row x 128-column tile variant
ROWS_PER_BLOCK = 4       # row-wise kernels: one row per 64-lane wave, 4 waves per block


def _cdiv(a, b):
    return -(-a // b)


# ----------------------------------------------------------------------------- grids
def grid_of(name, args):
    if name == "saxpy":
        return (_cdiv(args["n"], THREADS), 1, 1)
    if name == "reduce_sum":
        return (_cdiv(args["n"], REDUCE_BLOCK), 1, 1)
    if name == "reduce_final":
        return (1, 1, 1)
    if name == "gemm_bf16":
        return (_cdiv(args["n"], GEMM_TILE), _cdiv(args["m"], GEMM_TILE), args.get("batch", 1))
    if name == "gemm_bf16_small":
        return (_cdiv(args["n"], GEMM_SMALL_TILE), _cdiv(args["m"], GEMM_SMALL_TILE),
                args.get("batch", 1))
    if name == "gemm_bf16_n128":
        return (_cdiv(args["n"], GEMM_N128_COLS), _cdiv(args["m"], GEMM_TILE), args.get("batch", 1))
    if name == "gemv_bf16":
        return (_cdiv(args["n"], ROWS_PER_BLOCK), 1, 1)
    if name in ("softmax_f32", "layernorm_f32"):
        return (_cdiv(args["rows"], ROWS_PER_BLOCK), 1, 1)
    if name == "attn_decode_bf16":
        return (args["heads"], 1, 1)
    raise KeyError(name)


# ----------------------------------------------------------------------------- bodies
def _saxpy(b, grid, a):
    # y[i] = alpha * x[i] + y[i] for the block's 256 consecutive elements, guard i < n
    lo = b[0] * THREADS
    hi = min(lo + THREADS, a["n"])
    if hi <= lo:
        return
    x = a["x"][lo:hi].astype(np.float64)
    y = a["y"][lo:hi].astype(np.float64)
    a["y"][lo:hi] = (float(a["a"]) * x + y).astype(np.float32)


def _reduce_sum(b, grid, a):
    # partial[bx] = sum of the block's 4096 consecutive elements (ragged tail allowed)
    lo = b[0] * REDUCE_BLOCK
    hi = min(lo + REDUCE_BLOCK, a["n"])
    s = math.fsum(a["x"][lo:hi].astype(np.float64)) if hi > lo else 0.0
    a["partial"][b[0]] = np.float32(s)


def _reduce_final(b, grid, a):
    # total = sum of all per-block partials, carried and stored in fp64
    a["total"][0] = math.fsum(a["partial"][: a["count"]].astype(np.float64))


def _gemm_tile(b, grid, a, tile, tile_cols=None):
    # C[z, r0:r1, c0:c1] = A[z, r0:r1, :] . Bt[z, c0:c1, :]^T, bf16 in, bf16 out
    bx, by, bz = b
    tile_cols = tile if tile_cols is None else tile_cols
    r0, r1 = by * tile, min((by + 1) * tile, a["m"])
    c0, c1 = bx * tile_cols, min((bx + 1) * tile_cols, a["n"])
    if r1 <= r0 or c1 <= c0:
        return
    A = bf16.decode(a["A"][bz, r0:r1, :])
    Bt = bf16.decode(a["Bt"][bz, c0:c1, :])
    a["C"][bz, r0:r1, c0:c1] = bf16.encode(A @ Bt.T)


def _gemm(b, grid, a):
    _gemm_tile(b, grid, a, GEMM_TILE)


def _gemm_small(b, grid, a):
    _gemm_tile(b, grid, a, GEMM_SMALL_TILE)


def _gemm_n128(b, grid, a):
    _gemm_tile(b, grid, a, GEMM_TILE, GEMM_N128_COLS)


def _gemv(b, grid, a):
    # y[r] = sum_k x[k] * W[r, k] for the block's 4 rows
    r0, r1 = b[0] * ROWS_PER_BLOCK, min((b[0] + 1) * ROWS_PER_BLOCK, a["n"])
    if r1 <= r0:
        return
    x = bf16.decode(a["x"])
    W = bf16.decode(a["W"][r0:r1, :])
    a["y"][r0:r1] = bf16.encode(W @ x)


def _softmax(b, grid, a):
    # y[r, :] = exp(x[r, :] - max) / sum exp(x[r, :] - max) for the block's 4 rows
    r0, r1 = b[0] * ROWS_PER_BLOCK, min((b[0] + 1) * ROWS_PER_BLOCK, a["rows"])
    for r in range(r0, r1):
        x = a["x"][r, : a["cols"]].astype(np.float64)
        e = np.exp(x - x.max())
        a["y"][r, : a["cols"]] = (e / e.sum()).astype(np.float32)


def _layernorm(b, grid, a):
    # y = (x - mean) / sqrt(var + eps) * gamma + beta, biased variance, per row
    r0, r1 = b[0] * ROWS_PER_BLOCK, min((b[0] + 1) * ROWS_PER_BLOCK, a["rows"])
    g = a["gamma"].astype(np.float64)
    be = a["beta"].astype(np.float64)
    for r in range(r0, r1):
        x = a["x"][r, : a["cols"]].astype(np.float64)
        mu = x.mean()
        var = ((x - mu) ** 2).mean()
        a["y"][r, : a["cols"]] = ((x - mu) / math.sqrt(var + float(a["eps"])) * g + be).astype(
            np.float32)


def _attn_decode(b, grid, a):
    # one query per head: softmax(q . K^T / sqrt(dim)) . V over the cached tokens
    h = b[0]
    q = bf16.decode(a["q"][h])
    K = bf16.decode(a["K"][:, h, :])
    V = bf16.decode(a["V"][:, h, :])
    s = (K @ q) / math.sqrt(a["dim"])
    p = np.exp(s - s.max())
    p /= p.sum()
    a["out"][h] = bf16.encode(p @ V)


_BODIES = {
    "saxpy": _saxpy,
    "reduce_sum": _reduce_sum,
    "reduce_final": _reduce_final,
    "gemm_bf16": _gemm,
    "gemm_bf16_small": _gemm_small,
    "gemm_bf16_n128": _gemm_n128,
    "gemv_bf16": _gemv,
    "softmax_f32": _softmax,
    "layernorm_f32": _layernorm,
    "attn_decode_bf16": _attn_decode,
}


def exec_block(name, b, grid, args):
    _BODIES[name](b, grid, args)
