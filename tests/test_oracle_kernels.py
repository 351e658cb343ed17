"""Pins for the oracle's logical-block bodies: closed forms, invariants, special cases
that reduce to a library routine, and element-by-element brute force on tiny inputs."""
import math
import struct

import numpy as np
import pytest
import torch

import tally_inputs as TI
from oracle import bf16
from oracle import kernels as K
from oracle import schedules as S


def _bf(x):
    return TI.to_bf16_bits(np.asarray(x, dtype=np.float32))


def _one_bf16(bits):
    """Independent decode of one bf16 pattern through the struct module."""
    return struct.unpack("<f", struct.pack("<I", int(bits) << 16))[0]


# ------------------------------------------------------------------ bf16 storage
def test_bf16_known_patterns_and_ties():
    assert bf16.encode(np.array([1.0]))[0] == 0x3F80
    assert bf16.encode(np.array([-2.0]))[0] == 0xC000
    assert bf16.encode(np.array([1.0 + 2.0 ** -8]))[0] == 0x3F80       # tie -> even (down)
    assert bf16.encode(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 0x3F82   # tie -> even (up)
    assert bf16.encode(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 0x3F81
    assert bf16.decode(np.array([0x3F81], dtype=np.uint16))[0] == 1.0 + 2.0 ** -7


def test_bf16_matches_torch_cast():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000)).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (bf16.encode(x.astype(np.float64)) == want).all()
    assert (TI.to_bf16_bits(x) == want).all()
    back = torch.from_numpy(want.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert (bf16.decode(want) == back).all()


# ------------------------------------------------------------------ SAXPY
def test_saxpy_closed_form_and_ragged_tail():
    n = 1000                                   # 4 blocks, last one ragged (232 live threads)
    a = {"a": np.float32(1.5), "x": np.ones(n, np.float32), "y": np.full(n, 2, np.float32), "n": n}
    grid = K.grid_of("saxpy", a)
    assert grid == (4, 1, 1)
    S.run_native("saxpy", grid, a)
    assert (a["y"] == np.float32(3.5)).all()


def test_saxpy_random_and_schedule_independence():
    base = TI.saxpy_inputs(n=5000, config_index=0)
    want = (1.5 * base["x"].astype(np.float64) + base["y"].astype(np.float64)).astype(np.float32)
    grid = K.grid_of("saxpy", base)
    outs = []
    for mode in ("native", "sliced", "ptb", "ptb2"):
        a = dict(base, y=base["y"].copy())
        if mode == "native":
            cov = S.run_native("saxpy", grid, a)
        elif mode == "sliced":
            cov, _ = S.run_sliced("saxpy", grid, a, 3, preempt_after_slices=[2])
        elif mode == "ptb":
            cov, _ = S.run_ptb("saxpy", grid, a, 4, preempt_points=[3, 11], seed=1)
        else:
            cov, _ = S.run_ptb("saxpy", grid, a, 7, preempt_points=[1], seed=99)
        assert cov.exactly_once()
        outs.append(a["y"])
    for o in outs:
        assert (o.view(np.uint32) == want.view(np.uint32)).all()
    # an un-run block leaves its elements untouched: running twice must differ
    a = dict(base, y=base["y"].copy())
    S.run_naive_sliced("saxpy", grid, a, 5)
    assert not (a["y"] == want).all()


# ------------------------------------------------------------------ reduction
def test_reduce_all_ones_is_exact():
    n = 1 << 16
    a = {"x": np.ones(n, np.float32), "n": n, "partial": np.zeros(16, np.float32)}
    grid = K.grid_of("reduce_sum", a)
    assert grid == (16, 1, 1)
    S.run_native("reduce_sum", grid, a)
    assert (a["partial"] == 4096.0).all()
    f = {"partial": a["partial"], "count": 16, "total": np.zeros(1, np.float64)}
    S.run_native("reduce_final", (1, 1, 1), f)
    assert f["total"][0] == float(n)


def test_reduce_uniform_vs_numpy_and_clt():
    n = 4096 * 37 + 123                        # ragged last block
    x = TI.reduce_inputs(n=n, config_index=2)["x"]
    nb = K.grid_of("reduce_sum", {"n": n})[0]
    assert nb == 38
    a = {"x": x, "n": n, "partial": np.zeros(nb, np.float32)}
    cov, _ = S.run_sliced("reduce_sum", (nb, 1, 1), a, 8)
    assert cov.exactly_once()
    want = np.add.reduceat(x.astype(np.float64), np.arange(0, n, 4096))
    assert np.allclose(a["partial"], want, rtol=6e-8, atol=0)
    assert abs(a["partial"][-1] - x[37 * 4096:].astype(np.float64).sum()) < 1e-4
    f = {"partial": a["partial"], "count": nb, "total": np.zeros(1, np.float64)}
    S.run_native("reduce_final", (1, 1, 1), f)
    assert abs(f["total"][0] - np.sum(x, dtype=np.float64)) / n < 1e-7
    # mean of U(0,1) is 1/2 with standard error sqrt(1/12/n): stay within 6 sigma
    assert abs(f["total"][0] / n - 0.5) < 6 * math.sqrt(1 / 12 / n)


# ------------------------------------------------------------------ GEMM / GEMV
def test_gemm_identity_and_constant():
    m = n = k = 256
    eye = _bf(np.eye(256))[None]
    Bt = TI.normal_bf16(np.random.default_rng(5), (1, n, k), 1 / 64)
    a = {"A": eye, "Bt": Bt, "C": np.zeros((1, m, n), np.uint16), "m": m, "n": n, "k": k, "batch": 1}
    S.run_native("gemm_bf16", K.grid_of("gemm_bf16", a), a)
    assert (a["C"][0] == Bt[0].T).all()                     # I . B = B, bit for bit
    k = 4096
    ones = _bf(np.full((1, 256, k), 1 / 64))
    a = {"A": ones, "Bt": ones.copy(), "C": np.zeros((1, 256, 256), np.uint16),
         "m": 256, "n": 256, "k": k, "batch": 1}
    S.run_native("gemm_bf16", (1, 1, 1), a)
    assert (a["C"] == 0x3F80).all()                         # 4096 / 64^2 = 1 exactly


def test_gemm_elementwise_brute_force_rectangular_batched():
    # m, n, k all different and not multiples of the tile: catches transposed operands,
    # swapped tile axes and dropped edge handling
    m, n, k, batch = 300, 520, 72, 2
    g = TI.gemm_inputs(m, n, k, config_index=1, batch=batch)
    a = dict(g, C=np.zeros((batch, m, n), np.uint16))
    grid = K.grid_of("gemm_bf16", a)
    assert grid == (3, 2, 2)
    cov, _ = S.run_ptb("gemm_bf16", grid, a, 5, preempt_points=[4], seed=3)
    assert cov.exactly_once()
    rng = np.random.default_rng(0)
    for _ in range(40):
        z, i, j = int(rng.integers(batch)), int(rng.integers(m)), int(rng.integers(n))
        acc = 0.0
        for kk in range(k):
            acc += _one_bf16(g["A"][z, i, kk]) * _one_bf16(g["Bt"][z, j, kk])
        got = _one_bf16(a["C"][z, i, j])
        assert abs(got - acc) <= 2.0 ** -8 * abs(acc) + 1e-30
    # same result through the 32-wide tiling (each element written once either way)
    b = dict(g, C=np.zeros((batch, m, n), np.uint16))
    S.run_native("gemm_bf16_small", K.grid_of("gemm_bf16_small", b), b)
    assert (a["C"] == b["C"]).all()
    # and through the 256-row x 128-column tiling: grid (5, 2, 2), tile axes not interchangeable
    c = dict(g, C=np.zeros((batch, m, n), np.uint16))
    assert K.grid_of("gemm_bf16_n128", c) == (5, 2, 2)
    S.run_native("gemm_bf16_n128", K.grid_of("gemm_bf16_n128", c), c)
    assert (a["C"] == c["C"]).all()
    one = dict(g, C=np.zeros((batch, m, n), np.uint16))
    K.exec_block("gemm_bf16_n128", (1, 0, 1), (5, 2, 2), one)      # rows 0..255, cols 128..255
    touched = np.argwhere(one["C"] != 0)
    assert touched[:, 0].min() == 1 == touched[:, 0].max()
    assert touched[:, 1].max() <= 255 and 128 <= touched[:, 2].min() and touched[:, 2].max() <= 255
    # library cross-check: torch fp64 matmul of the decoded operands
    A64 = torch.from_numpy(bf16.decode(g["A"]))
    B64 = torch.from_numpy(bf16.decode(g["Bt"]))
    ref = torch.matmul(A64, B64.transpose(1, 2)).to(torch.float32).to(torch.bfloat16)
    assert (ref.view(torch.int16).numpy().view(np.uint16) == a["C"]).all()


def test_gemv_is_a_one_row_gemm_and_identity():
    g = TI.gemv_inputs(n=130, k=96, config_index=1)       # ragged last block (2 rows)
    a = dict(g, y=np.zeros(130, np.uint16))
    grid = K.grid_of("gemv_bf16", a)
    assert grid == (33, 1, 1)
    S.run_native("gemv_bf16", grid, a)
    gm = {"A": g["x"][None, None, :], "Bt": g["W"][None], "C": np.zeros((1, 1, 130), np.uint16),
          "m": 1, "n": 130, "k": 96, "batch": 1}
    S.run_native("gemm_bf16", K.grid_of("gemm_bf16", gm), gm)
    assert (gm["C"][0, 0] == a["y"]).all()
    eye = {"x": g["x"][:96], "W": _bf(np.eye(96)), "n": 96, "k": 96, "y": np.zeros(96, np.uint16)}
    S.run_native("gemv_bf16", K.grid_of("gemv_bf16", eye), eye)
    assert (eye["y"] == g["x"][:96]).all()


# ------------------------------------------------------------------ softmax / LayerNorm
def test_softmax_closed_forms_and_invariants():
    x = np.zeros((6, 128), np.float32)
    x[1, :] = 7.25                                          # constant row -> uniform
    x[2, :2] = [0.0, math.log(3.0)]
    x[2, 2:] = -1e4                                         # two live entries -> 1/4, 3/4
    x[3] = TI.rows_f32(1, 128, 1.0)[0]
    x[4] = x[3] + 100.0                                     # shift invariance
    x[5] = TI.rows_f32(1, 128, 30.0, stream=9)[0]           # large magnitudes: no overflow
    a = {"x": x, "y": np.zeros_like(x), "rows": 6, "cols": 128}
    grid = K.grid_of("softmax_f32", a)
    assert grid == (2, 1, 1)
    S.run_native("softmax_f32", grid, a)
    y = a["y"]
    assert np.allclose(y.sum(axis=1, dtype=np.float64), 1.0, atol=1e-6)
    assert np.allclose(y[1], 1 / 128, rtol=1e-7)
    assert np.allclose(y[2, :2], [0.25, 0.75], rtol=1e-6) and (y[2, 2:] == 0).all()
    assert np.allclose(y[3], y[4], rtol=1e-5)
    assert np.isfinite(y).all() and (y >= 0).all()
    ref = torch.softmax(torch.from_numpy(x).double(), dim=1).float().numpy()
    assert np.allclose(y, ref, rtol=1e-6, atol=1e-30)


def test_layernorm_closed_form_and_invariants():
    li = TI.layernorm_inputs(5, 768)
    a = dict(li, y=np.zeros_like(li["x"]))
    S.run_native("layernorm_f32", K.grid_of("layernorm_f32", a), a)
    ref = torch.nn.functional.layer_norm(
        torch.from_numpy(li["x"]).double(), (768,), torch.from_numpy(li["gamma"]).double(),
        torch.from_numpy(li["beta"]).double(), eps=float(li["eps"])).float().numpy()
    assert np.allclose(a["y"], ref, rtol=1e-6, atol=1e-7)
    # gamma = 1, beta = 0, eps = 0: zero mean, unit (biased) variance
    b = {"x": li["x"], "gamma": np.ones(768, np.float32), "beta": np.zeros(768, np.float32),
         "eps": np.float32(0), "rows": 5, "cols": 768, "y": np.zeros_like(li["x"])}
    S.run_native("layernorm_f32", K.grid_of("layernorm_f32", b), b)
    assert np.allclose(b["y"].mean(axis=1, dtype=np.float64), 0, atol=1e-6)
    assert np.allclose(b["y"].astype(np.float64).var(axis=1), 1, atol=1e-5)
    # [1,2,3,4]: mean 2.5, variance 1.25
    c = {"x": np.array([[1, 2, 3, 4]], np.float32), "gamma": np.array([1, 1, 2, 1], np.float32),
         "beta": np.array([0, 0.5, 0, 0], np.float32), "eps": np.float32(0), "rows": 1, "cols": 4,
         "y": np.zeros((1, 4), np.float32)}
    S.run_native("layernorm_f32", (1, 1, 1), c)
    s = math.sqrt(1.25)
    assert np.allclose(c["y"][0], [-1.5 / s, -0.5 / s + 0.5, 2 * 0.5 / s, 1.5 / s], rtol=1e-6)


# ------------------------------------------------------------------ decode attention
def test_attn_decode_special_cases():
    T, H, D = 64, 3, 128
    at = TI.attn_decode_inputs(T, H, D, scale=1.0)
    # identical keys -> uniform weights -> output is the mean of V
    a = dict(at, out=np.zeros((H, D), np.uint16))
    a["K"] = np.broadcast_to(at["K"][:1], at["K"].shape).copy()
    S.run_native("attn_decode_bf16", K.grid_of("attn_decode_bf16", a), a)
    want = bf16.encode(bf16.decode(at["V"]).mean(axis=0))
    assert (a["out"] == want).all()
    # two tokens: weights are a logistic function of the scaled score difference
    q = _bf(np.ones((1, D)))
    Kc = _bf(np.stack([np.full((1, D), 0.25), np.zeros((1, D))]))        # scores 32, 0
    Vc = _bf(np.stack([np.ones((1, D)), -np.ones((1, D))]))
    b = {"q": q, "K": Kc, "V": Vc, "tokens": 2, "heads": 1, "dim": D,
         "out": np.zeros((1, D), np.uint16)}
    S.run_native("attn_decode_bf16", (1, 1, 1), b)
    p0 = 1 / (1 + math.exp(-32 / math.sqrt(D)))
    assert np.allclose(bf16.decode(b["out"]), 2 * p0 - 1, rtol=2.0 ** -8)
    # library cross-check
    c = dict(at, out=np.zeros((H, D), np.uint16))
    S.run_native("attn_decode_bf16", K.grid_of("attn_decode_bf16", c), c)
    qq = torch.from_numpy(bf16.decode(at["q"]))[:, None, :]
    KK = torch.from_numpy(bf16.decode(at["K"])).permute(1, 0, 2)
    VV = torch.from_numpy(bf16.decode(at["V"])).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(qq, KK, VV)[:, 0, :]
    assert (bf16.encode(ref.numpy()) == c["out"]).all()
