"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws random numbers and packs them into arrays.  It holds none
of the scheduling method's arithmetic and none of the workload kernels' math: the
CPU oracle and the HIP path both receive the *same bits* produced here and never
see each other's code.

Generator: NumPy PCG64, seed = BASE_SEED + config index.  bf16 tensors are
returned as uint16 bit patterns (round-to-nearest-even from fp32), because that is
the storage format both sides consume.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 241007381


def rng_for(config_index: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([BASE_SEED + config_index, stream]))


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even (storage packing)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def normal_f32(rng, shape, scale=1.0):
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)).astype(np.float32)


def normal_bf16(rng, shape, scale=1.0):
    return to_bf16_bits(normal_f32(rng, shape, scale))


def uniform_f32(rng, shape):
    return rng.random(shape, dtype=np.float32)


# ---------------------------------------------------------------------------
# Workload recipes (shapes follow the five benchmark configurations)
# ---------------------------------------------------------------------------

def saxpy_inputs(n=1 << 20, config_index=0):
    """x, y ~ N(0,1) fp32, a = 1.5."""
    rng = rng_for(config_index)
    return {"a": np.float32(1.5), "x": normal_f32(rng, n), "y": normal_f32(rng, n), "n": n}


def preempt_points(total_blocks, count=3, config_index=0):
    """`count` distinct sorted counter values in [1, total_blocks-1]."""
    rng = rng_for(config_index, stream=1)
    count = min(count, max(total_blocks - 1, 0))
    if count == 0:
        return []
    pts = rng.choice(np.arange(1, total_blocks), size=count, replace=False)
    return sorted(int(p) for p in pts)


def gemm_inputs(m=4096, n=4096, k=4096, scale=1.0 / 64.0, config_index=1, batch=1):
    """A[batch,m,k] and Bt[batch,n,k] (B stored K-contiguous) as bf16 bits, ~N(0,1)*scale."""
    rng = rng_for(config_index)
    a = normal_bf16(rng, (batch, m, k), scale)
    bt = normal_bf16(rng, (batch, n, k), scale)
    return {"A": a, "Bt": bt, "m": m, "n": n, "k": k, "batch": batch}


def gemv_inputs(n=4096, k=4096, scale=1.0 / 64.0, config_index=1):
    """x[k], W[n,k] (each output is a dot product over one K-contiguous row)."""
    rng = rng_for(config_index, stream=2)
    return {"x": normal_bf16(rng, k, scale), "W": normal_bf16(rng, (n, k), scale), "n": n, "k": k}


def reduce_inputs(n=1 << 28, config_index=2):
    rng = rng_for(config_index)
    return {"x": uniform_f32(rng, n), "n": n}


def rows_f32(rows, cols, scale=0.02, config_index=3, stream=0):
    rng = rng_for(config_index, stream)
    return normal_f32(rng, (rows, cols), scale)


def layernorm_inputs(rows, cols, scale=0.02, config_index=3, stream=3):
    rng = rng_for(config_index, stream)
    return {
        "x": normal_f32(rng, (rows, cols), scale),
        "gamma": (1.0 + normal_f32(rng, cols, scale)).astype(np.float32),
        "beta": normal_f32(rng, cols, scale),
        "eps": np.float32(1e-5),
        "rows": rows,
        "cols": cols,
    }


def attn_decode_inputs(tokens=2048, heads=32, dim=128, scale=0.02, config_index=4):
    """q[heads,dim], K/V cache [tokens,heads,dim], bf16 bits."""
    rng = rng_for(config_index, stream=4)
    return {
        "q": normal_bf16(rng, (heads, dim), scale),
        "K": normal_bf16(rng, (tokens, heads, dim), scale),
        "V": normal_bf16(rng, (tokens, heads, dim), scale),
        "tokens": tokens, "heads": heads, "dim": dim,
    }


def rolled_blocks_bf16(rng, blocks, rows, cols, scale):
    """A [blocks, rows, cols] bf16 tensor for operands too large to draw element by element
    in a test: one seeded N(0, scale) block of rows x cols, and for block z a copy rolled by
    (13 z + 1) rows and (29 z + 5) columns, so that the blocks differ from one another while
    every element keeps the distribution of the first."""
    base = normal_bf16(rng, (rows, cols), scale)
    out = np.empty((blocks, rows, cols), dtype=np.uint16)
    for z in range(blocks):
        out[z] = np.roll(base, (13 * z + 1, 29 * z + 5), axis=(0, 1))
    return out


def poisson_arrivals_us(rate_per_s, count, config_index, stream=7):
    """Open-loop arrival times (microseconds from t0) of a Poisson process."""
    rng = rng_for(config_index, stream)
    gaps = rng.exponential(1e6 / rate_per_s, size=count)
    return np.cumsum(gaps)


def bursty_arrivals_us(mean_rate_per_s, count, config_index, burst=50.0, p_on=0.02,
                       mean_segment_us=20000.0, stream=8):
    """Open-loop arrivals of an on/off-modulated Poisson process with the given mean rate:
    time is cut into segments of exponential length; a segment is "on" with probability
    p_on and then has `burst` times the arrival rate of an "off" segment (load spikes of
    tens of times the average, as production inference traces show)."""
    rng = rng_for(config_index, stream)
    rate_off = mean_rate_per_s / (1.0 - p_on + p_on * burst)
    out, t = [], 0.0
    while len(out) < count:
        seg = rng.exponential(mean_segment_us)
        rate = rate_off * (burst if rng.random() < p_on else 1.0)
        u = t
        while True:
            u += rng.exponential(1e6 / rate)
            if u > t + seg or len(out) >= count:
                break
            out.append(u)
        t += seg
    return np.asarray(out[:count], dtype=np.float64)


def periodic_arrivals_us(period_us, count):
    return np.arange(1, count + 1, dtype=np.float64) * period_us
