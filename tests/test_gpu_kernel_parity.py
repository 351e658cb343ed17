"""GPU parity of the workload kernels (GEMM, GEMV, softmax, LayerNorm, decode attention) in
their native and transformed forms against the CPU oracle, element by element, and on
sampled tiles at the full benchmark sizes."""
import numpy as np
import pytest

import tally_inputs as TI
from oracle import kernels as OK
from oracle import schedules as OS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2410_07381_amd.binding as B
    assert torch.cuda.is_available(), "these tests need the MI355X"
    hi, be = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(hi, be)
    yield B, ctx, torch
    ctx.close()


def _run_form(B, ctx, torch, kernel, form):
    if form == "native":
        ctx.launch_native(kernel)
    elif form == "native_hi":
        ctx.launch_native(kernel, hi=True)
    else:
        if form == "sliced":
            job = ctx.launch_sliced(kernel, 3)
        elif form == "ptb":
            job = ctx.launch_ptb(kernel, 5)
        else:                                             # preempted half way, then resumed
            job = ctx.launch_ptb(kernel, 3, chunk=2, stop_at=max(1, kernel.total_blocks // 2))
            job.wait()
            job.resume()
        assert job.wait() == B.JOB_COMPLETE
        job.free()
    torch.cuda.synchronize()


FORMS = ["native", "sliced", "ptb", "ptb_preempted"]


# ------------------------------------------------------------------ GEMM, 256-wide tiles
@pytest.mark.parametrize("form", FORMS)
def test_gemm_bf16_forms(env, form):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    m, n, k, batch = 512, 768, 320, 2                    # 3 x 2 x 2 tiles, 5 k-steps
    g = TI.gemm_inputs(m, n, k, config_index=1, batch=batch)
    a = dict(g, C=np.zeros((batch, m, n), np.uint16))
    OS.run_native("gemm_bf16", OK.grid_of("gemm_bf16", a), a)
    A, Bt, Cd = dev(g["A"]), dev(g["Bt"]), dev(np.zeros((batch, m, n), np.uint16))
    torch.cuda.synchronize()
    kern = B.gemm_bf16(A, Bt, Cd)
    assert kern.grid == (3, 2, 2)
    _run_form(B, ctx, torch, kern, form)
    assert_bf16_close(host(Cd), a["C"])


@pytest.mark.parametrize("k", [32, 64, 96, 128])
@pytest.mark.parametrize("form", ["native", "ptb"])
def test_gemm_short_k(env, k, form):
    """One to four k-steps: fewer than the LDS ring has stages (prologue and drain paths)."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    m, n = 256, 512
    g = TI.gemm_inputs(m, n, k, config_index=3, scale=0.25)
    a = dict(g, C=np.zeros((1, m, n), np.uint16))
    OS.run_native("gemm_bf16", OK.grid_of("gemm_bf16", a), a)
    A, Bt, Cd = dev(g["A"]), dev(g["Bt"]), dev(np.zeros((1, m, n), np.uint16))
    torch.cuda.synchronize()
    _run_form(B, ctx, torch, B.gemm_bf16(A, Bt, Cd), form)
    assert_bf16_close(host(Cd), a["C"])


def test_gemm_training_step_shapes(env):
    """Shapes of the transformer-layer step: attention scores (batched, K = 128, 2048 x 2048
    outputs per batch) and the second FFN product (K = 16384), persistent workers; the
    oracle recomputes whole batches / tiles."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    g = TI.gemm_inputs(2048, 2048, 128, config_index=3, batch=3, scale=0.25)
    A, Bt = dev(g["A"]), dev(g["Bt"])
    Cd = torch.zeros((3, 2048, 2048), dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    kern = B.gemm_bf16(A, Bt, Cd)
    assert kern.grid == (8, 8, 3)
    job = ctx.launch_ptb(kern, 256)
    assert job.wait() == B.JOB_COMPLETE
    job.free()
    a = dict(g, C=np.zeros((3, 2048, 2048), np.uint16))
    OS.run_native("gemm_bf16", OK.grid_of("gemm_bf16", a), a)
    assert_bf16_close(host(Cd), a["C"])
    g = TI.gemm_inputs(512, 256, 16384, config_index=3, scale=1.0 / 128.0)
    A, Bt = dev(g["A"]), dev(g["Bt"])
    Cd = torch.zeros((1, 512, 256), dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    job = ctx.launch_ptb(B.gemm_bf16(A, Bt, Cd), 256)
    assert job.wait() == B.JOB_COMPLETE
    job.free()
    a = dict(g, C=np.zeros((1, 512, 256), np.uint16))
    OS.run_native("gemm_bf16", OK.grid_of("gemm_bf16", a), a)
    assert_bf16_close(host(Cd), a["C"])


@pytest.mark.parametrize("form", FORMS)
def test_gemm_n128_forms(env, form):
    """256-row x 128-column tiles (n a multiple of 128 only): 3 x 2 x 2 tiles, 6 k-steps."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    m, n, k, batch = 512, 384, 192, 2
    g = TI.gemm_inputs(m, n, k, config_index=3, batch=batch, scale=0.125)
    a = dict(g, C=np.zeros((batch, m, n), np.uint16))
    OS.run_native("gemm_bf16_n128", OK.grid_of("gemm_bf16_n128", a), a)
    A, Bt, Cd = dev(g["A"]), dev(g["Bt"]), dev(np.zeros((batch, m, n), np.uint16))
    torch.cuda.synchronize()
    kern = B.gemm_bf16(A, Bt, Cd, n128=True)
    assert kern.grid == (3, 2, 2)
    _run_form(B, ctx, torch, kern, form)
    assert_bf16_close(host(Cd), a["C"])


@pytest.mark.parametrize("k", [32, 96, 2048])
def test_gemm_n128_attention_value_shape(env, k):
    """The P.V product of the training-like step: 2048 x 128 outputs per batch entry."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    m, n, batch = 2048, 128, 2
    g = TI.gemm_inputs(m, n, k, config_index=3, batch=batch, scale=0.05)
    a = dict(g, C=np.zeros((batch, m, n), np.uint16))
    OS.run_native("gemm_bf16_n128", OK.grid_of("gemm_bf16_n128", a), a)
    A, Bt, Cd = dev(g["A"]), dev(g["Bt"]), dev(np.zeros((batch, m, n), np.uint16))
    torch.cuda.synchronize()
    kern = B.gemm_bf16(A, Bt, Cd, n128=True)
    assert kern.grid == (1, 8, 2)
    job = ctx.launch_ptb(kern, 256)
    assert job.wait() == B.JOB_COMPLETE
    job.free()
    assert_bf16_close(host(Cd), a["C"])


@pytest.mark.parametrize("variant", ["big", "n128", "small"])
def test_gemm_padded_leading_dimensions(env, variant):
    """Operands stored with rows longer than k (views of padded buffers, batch pitch larger
    than the matrix): same result as the oracle gets from the unpadded arrays."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    m, n, k, batch = (512, 512, 160, 2) if variant == "big" else ((256, 384, 96, 2) if variant == "n128"
                                                                    else (100, 70, 64, 2))
    name = {"big": "gemm_bf16", "n128": "gemm_bf16_n128", "small": "gemm_bf16_small"}[variant]
    g = TI.gemm_inputs(m, n, k, config_index=3, batch=batch, scale=0.125)
    a = dict(g, C=np.zeros((batch, m, n), np.uint16))
    OS.run_native(name, OK.grid_of(name, a), a)
    Ap = torch.full((batch, m + 3, k + 24), 0x7FC0, dtype=torch.int16, device="cuda")   # NaN padding
    Bp = torch.full((batch, n + 1, k + 8), 0x7FC0, dtype=torch.int16, device="cuda")
    Ap[:, :m, :k] = dev(g["A"])
    Bp[:, :n, :k] = dev(g["Bt"])
    Cd = torch.zeros((batch, m, n), dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    kern = B.gemm_bf16(Ap[:, :m, :k], Bp[:, :n, :k], Cd, small=(variant == "small"),
                       n128=(variant == "n128"))
    job = ctx.launch_ptb(kern, 7)
    assert job.wait() == B.JOB_COMPLETE
    job.free()
    assert_bf16_close(host(Cd), a["C"])
    bad = torch.zeros((1, 256, 256 + 4), dtype=torch.int16, device="cuda")              # pitch not a multiple of 8
    with pytest.raises(B.TallyError):
        B.gemm_bf16(bad[:, :, :256], bad[:, :, :256], torch.zeros((1, 256, 256), dtype=torch.int16, device="cuda"))


def test_gemm_rejects_unaligned_output(env):
    B, ctx, torch = env
    A = torch.zeros((1, 256, 64), dtype=torch.int16, device="cuda")
    Cbuf = torch.zeros(256 * 256 + 8, dtype=torch.int16, device="cuda")
    with pytest.raises(B.TallyError):
        B.gemm_bf16(A, A, Cbuf[1:1 + 256 * 256].view(1, 256, 256))


def test_gemm_identity_is_exact(env):
    B, ctx, torch = env
    from gpu_util import dev, host
    eye = TI.to_bf16_bits(np.eye(256, dtype=np.float32))[None]
    Bt = TI.normal_bf16(np.random.default_rng(5), (1, 512, 256), 1 / 64)
    A, Btd, Cd = dev(eye), dev(Bt), dev(np.zeros((1, 256, 512), np.uint16))
    torch.cuda.synchronize()
    ctx.launch_native(B.gemm_bf16(A, Btd, Cd))
    torch.cuda.synchronize()
    assert (host(Cd)[0] == Bt[0].T).all()                # I . B = B bit for bit


def test_gemm_cfg1_full_size_sampled_tiles(env):
    """M = N = K = 4096 in persistent-worker form with 256 workers (the benchmark's launch
    configuration); the oracle recomputes a seeded sample of whole 256x256 tiles."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    g = TI.gemm_inputs(4096, 4096, 4096, config_index=1)
    A, Bt = dev(g["A"]), dev(g["Bt"])
    Cd = torch.zeros((1, 4096, 4096), dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    kern = B.gemm_bf16(A, Bt, Cd)
    assert kern.grid == (16, 16, 1)
    job = ctx.launch_ptb(kern, 256, coverage=True)
    assert job.wait() == B.JOB_COMPLETE
    rec = job.coverage()
    job.free()
    assert (rec["count"] == 1).all()
    idx = np.arange(256)
    assert (rec["bx"] == idx % 16).all() and (rec["by"] == idx // 16).all()
    got = host(Cd)
    rng = np.random.default_rng(11)
    for t in [0, 255] + [int(v) for v in rng.integers(1, 255, 3)]:
        bx, by = t % 16, t // 16
        a = dict(g, C=np.zeros((1, 4096, 4096), np.uint16))
        OK.exec_block("gemm_bf16", (bx, by, 0), (16, 16, 1), a)
        r, c = slice(by * 256, by * 256 + 256), slice(bx * 256, bx * 256 + 256)
        assert_bf16_close(got[0, r, c], a["C"][0, r, c])
    # all-ones / 64: every output is exactly 1 (property that holds at any size)
    ones = TI.to_bf16_bits(np.full((1, 4096, 4096), 1 / 64, np.float32))
    A1 = dev(ones)
    torch.cuda.synchronize()
    ctx.launch_native(B.gemm_bf16(A1, A1, Cd))
    torch.cuda.synchronize()
    assert (host(Cd) == 0x3F80).all()


# ------------------------------------------------------------------ GEMM, 32-wide ragged tiles
@pytest.mark.parametrize("form", FORMS)
def test_gemm_small_forms(env, form):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    m, n, k, batch = 300, 520, 96, 2
    g = TI.gemm_inputs(m, n, k, config_index=3, batch=batch)
    a = dict(g, C=np.zeros((batch, m, n), np.uint16))
    OS.run_native("gemm_bf16_small", OK.grid_of("gemm_bf16_small", a), a)
    A, Bt, Cd = dev(g["A"]), dev(g["Bt"]), dev(np.zeros((batch, m, n), np.uint16))
    torch.cuda.synchronize()
    _run_form(B, ctx, torch, B.gemm_bf16(A, Bt, Cd, small=True), form)
    assert_bf16_close(host(Cd), a["C"])


# ------------------------------------------------------------------ GEMV
@pytest.mark.parametrize("n,k,form", [(130, 96, "native"), (130, 96, "ptb_preempted"),
                                      (4096, 4096, "native_hi"), (4096, 11008, "native_hi"),
                                      (11008, 4096, "native_hi"), (1000, 2056, "sliced"),
                                      # the original form takes a row in batches of eight, then four
                                      # loads per lane, then singles: rows shorter than a batch, fewer
                                      # rows than a workgroup has waves, ragged ends of every loop
                                      (5, 8, "native"), (3, 520, "native_hi"), (1031, 4104, "native"),
                                      (300, 11264, "native_hi"), (37, 11272, "native")])
def test_gemv(env, n, k, form):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    g = TI.gemv_inputs(n=n, k=k, scale=1 / 64 if k == 4096 and n == 4096 else 0.02, config_index=1)
    a = dict(g, y=np.zeros(n, np.uint16))
    OS.run_native("gemv_bf16", OK.grid_of("gemv_bf16", a), a)
    x, W, y = dev(g["x"]), dev(g["W"]), dev(np.zeros(n, np.uint16))
    torch.cuda.synchronize()
    _run_form(B, ctx, torch, B.gemv_bf16(x, W, y), form)
    assert_bf16_close(host(y), a["y"])


# ------------------------------------------------------------------ softmax / LayerNorm
@pytest.mark.parametrize("rows,cols,form", [(37, 2048, "native"), (37, 2048, "ptb_preempted"),
                                            (37, 2048, "sliced"), (1536, 128, "native_hi"),
                                            (9, 8192, "ptb"), (5, 100, "native"),
                                            (3, 4096, "native")])
def test_softmax(env, rows, cols, form):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_close_rel
    xs = TI.rows_f32(rows, cols, scale=2.0, config_index=3)
    xs[0, :] = 0.25                                       # constant row
    xs[rows - 1, 0] = 60.0                                # one dominant entry
    a = {"x": xs, "y": np.zeros_like(xs), "rows": rows, "cols": cols}
    OS.run_native("softmax_f32", OK.grid_of("softmax_f32", a), a)
    x, y = dev(xs), dev(np.zeros_like(xs))
    torch.cuda.synchronize()
    _run_form(B, ctx, torch, B.softmax_f32(x, y), form)
    got = host(y)
    assert_close_rel(got, a["y"], 1e-5, 1e-7)
    assert np.allclose(got.sum(axis=1, dtype=np.float64), 1.0, atol=1e-5)


@pytest.mark.parametrize("rows,cols,form", [(41, 4096, "native"), (41, 4096, "ptb_preempted"),
                                            (41, 4096, "sliced"), (128, 768, "native_hi"),
                                            (6, 8192, "ptb"), (5, 100, "native")])
def test_layernorm(env, rows, cols, form):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_close_rel
    li = TI.layernorm_inputs(rows, cols, scale=1.0)
    a = dict(li, y=np.zeros_like(li["x"]))
    OS.run_native("layernorm_f32", OK.grid_of("layernorm_f32", a), a)
    x, g, b, y = dev(li["x"]), dev(li["gamma"]), dev(li["beta"]), dev(np.zeros_like(li["x"]))
    torch.cuda.synchronize()
    _run_form(B, ctx, torch, B.layernorm_f32(x, g, b, y, li["eps"]), form)
    assert_close_rel(host(y), a["y"], 1e-5, 2e-6)


# ------------------------------------------------------------------ decode attention
@pytest.mark.parametrize("tokens,heads,scale", [(2048, 32, 0.02), (777, 3, 1.0), (5, 2, 1.0)])
def test_attn_decode(env, tokens, heads, scale):
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    at = TI.attn_decode_inputs(tokens, heads, 128, scale=scale)
    a = dict(at, out=np.zeros((heads, 128), np.uint16))
    OS.run_native("attn_decode_bf16", OK.grid_of("attn_decode_bf16", a), a)
    q, Kc, Vc = dev(at["q"]), dev(at["K"]), dev(at["V"])
    out = dev(np.zeros((heads, 128), np.uint16))
    scratch = torch.zeros(B.attn_decode_scratch_bytes(heads), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    kern = B.attn_decode_bf16(q, Kc, Vc, out, scratch)
    ctx.launch_native(kern, hi=True)
    torch.cuda.synchronize()
    assert_bf16_close(host(out), a["out"])
    # the scratch serves later calls as it is
    first = host(out).copy()
    for _ in range(3):
        out.zero_()
        ctx.launch_native(kern, hi=True)
    torch.cuda.synchronize()
    assert (host(out) == first).all()


def test_attn_decode_longest_cache(env):
    """16 splits x 2048 tokens is the longest cache one call takes; one token more is refused."""
    B, ctx, torch = env
    from gpu_util import dev, host, assert_bf16_close
    tokens, heads = 16 * 2048, 2
    at = TI.attn_decode_inputs(tokens, heads, 128, scale=0.5)
    a = dict(at, out=np.zeros((heads, 128), np.uint16))
    OS.run_native("attn_decode_bf16", OK.grid_of("attn_decode_bf16", a), a)
    q, Kc, Vc = dev(at["q"]), dev(at["K"]), dev(at["V"])
    out = dev(np.zeros((heads, 128), np.uint16))
    scratch = torch.zeros(B.attn_decode_scratch_bytes(heads), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    ctx.launch_native(B.attn_decode_bf16(q, Kc, Vc, out, scratch), hi=True)
    torch.cuda.synchronize()
    assert_bf16_close(host(out), a["out"])
    Kbig = torch.zeros((tokens + 1, heads, 128), dtype=torch.int16, device="cuda")
    with pytest.raises(B.TallyError):
        B.attn_decode_bf16(q, Kbig, Kbig, out, scratch)
