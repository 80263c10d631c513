"""GPU parity of every step of the hot path against the fp64 CPU checker, element by element,
through the C ABI.  Small shapes that still span several tiles and ragged tails, plus the
degenerate cases (one token, one position, one head)."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import stage_oracle as so
from tests.gpu_util import (TOL_ADAM, TOL_BF16, TOL_FP32, f32_dev, rand, rel_err, require_gpu, stream_ptr, to_dev,
                            to_host, torch_dtype)

pytestmark = pytest.mark.gpu

BF16, FP32 = si.DTYPE_BF16, si.DTYPE_FP32


def tol_of(dtype):
    return TOL_BF16 if dtype == BF16 else TOL_FP32


@pytest.fixture(scope="module")
def env():
    torch = require_gpu()
    import paper_2412_12636_amd as tm
    return torch, tm


# ------------------------------------------------------------------ linear maps
LINEAR_SHAPES = [
    (BF16, 300, 264, 200),     # ragged in every dimension, several 128-tiles
    (BF16, 512, 512, 256),     # exact 256-tiles
    (BF16, 1, 8, 8),           # one token
    (BF16, 1000, 136, 72),     # tall, K tail of 8
    (FP32, 70, 72, 40),
    (FP32, 256, 256, 64),
]


@pytest.mark.parametrize("dtype,T,N,K", LINEAR_SHAPES)
def test_linear_fwd_dgrad_wgrad(env, dtype, T, N, K):
    torch, tm = env
    print(f"linear dtype={dtype} T={T} N={N} K={K}", flush=True)
    rng = np.random.default_rng(T * 7 + N)
    x, w = rand(rng, (T, K), 1.0, dtype), rand(rng, (N, K), 0.05, dtype)
    bias, res = rand(rng, (N,), 0.5, dtype), rand(rng, (T, N), 1.0, dtype)
    dy = rand(rng, (T, N), 0.1, dtype)
    td = torch_dtype(torch, dtype)
    xd, wd, bd, rd, dyd = (to_dev(torch, a, dtype) for a in (x, w, bias, res, dy))
    s = stream_ptr(torch)
    tol = tol_of(dtype)

    y = torch.empty((T, N), dtype=td, device="cuda")
    tm.tm_op_linear_fwd(dtype, T, N, K, xd, wd, bd, rd, y, s)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + bias + res
    assert rel_err(to_host(y), ref) <= tol
    y2 = torch.empty((T, N), dtype=td, device="cuda")
    tm.tm_op_linear_fwd(dtype, T, N, K, xd, wd, None, None, y2, s)
    assert rel_err(to_host(y2), x.astype(np.float64) @ w.astype(np.float64).T) <= tol

    dx = torch.empty((T, K), dtype=td, device="cuda")
    tm.tm_op_linear_dgrad(dtype, T, N, K, dyd, wd, dx, s)
    assert rel_err(to_host(dx), dy.astype(np.float64) @ w.astype(np.float64)) <= tol

    g0 = rng.standard_normal((N, K)).astype(np.float32)
    dw = f32_dev(torch, g0)
    tm.tm_op_linear_wgrad(dtype, T, N, K, dyd, xd, dw, 1, s)
    ref = g0.astype(np.float64) + dy.astype(np.float64).T @ x.astype(np.float64)
    # fp32 accumulation of exact products: far tighter than the storage tolerance
    assert rel_err(to_host(dw), ref) <= 1e-5


def test_every_tile_configuration_gives_the_same_bits_and_matches_the_checker(env):
    """Each tile configuration in turn is forced on the three products of a linear map (ragged edges, several tiles of
    the largest shape, all dimensions multiples of 64 so that the pipelined kernel runs): results equal the checker's
    within tolerance and equal the first configuration's bit for bit."""
    torch, tm = env
    T, N, K = 712, 584, 448
    rng = np.random.default_rng(11)
    x, w = rand(rng, (T, K), 1.0, BF16), rand(rng, (N, K), 0.05, BF16)
    bias, res, dy = rand(rng, (N,), 0.5, BF16), rand(rng, (T, N), 1.0, BF16), rand(rng, (T, N), 0.1, BF16)
    xd, wd, bd, rd, dyd = (to_dev(torch, a, BF16) for a in (x, w, bias, res, dy))
    dy64 = dy.astype(np.float64)
    s = stream_ptr(torch)
    ref_y = x.astype(np.float64) @ w.astype(np.float64).T + bias + res
    first = None
    n = tm.tm_gemm_config_count()
    assert n >= 13
    try:
        for c in range(n):
            print(f"tile configuration {c}", flush=True)
            tm.tm_gemm_force_config(c)
            y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
            dx = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
            dw = torch.empty((N, K), dtype=torch.float32, device="cuda")
            tm.tm_op_linear_fwd(BF16, T, N, K, xd, wd, bd, rd, y, s)
            tm.tm_op_linear_dgrad(BF16, T, N, K, dyd, wd, dx, s)
            tm.tm_op_linear_wgrad(BF16, T, N, K, dyd, xd, dw, 0, s)
            tm.tm_op_linear_wgrad(BF16, T, N, K, dyd, xd, dw, 1, s)      # adds the same product again
            torch.cuda.synchronize()
            assert rel_err(to_host(y), ref_y) <= TOL_BF16
            assert rel_err(to_host(dx), dy64 @ w.astype(np.float64)) <= TOL_BF16
            assert rel_err(to_host(dw), 2.0 * (dy64.T @ x.astype(np.float64))) <= 1e-5
            if first is None:
                first = (y, dx, dw)
            else:
                assert torch.equal(y, first[0]) and torch.equal(dx, first[1]) and torch.equal(dw, first[2]), c
    finally:
        tm.tm_gemm_force_config(-1)
    with pytest.raises(tm.TmError):
        tm.tm_gemm_force_config(n)


def test_input_gradient_with_split_reduction(env):
    """dx = dy W with few output tiles and a long reduction: with scratch the reduction is split (the size
    query says so), the result meets the same tolerance against the definition and is reproducible; without
    scratch the call is the plain product."""
    torch, tm = env
    T, N, K = 300, 4096, 264                     # reduction over N = 4096, output 300 x 264: six tiles
    rng = np.random.default_rng(21)
    dy, w = rand(rng, (T, N), 0.1, BF16), rand(rng, (N, K), 0.05, BF16)
    dyd, wd = to_dev(torch, dy, BF16), to_dev(torch, w, BF16)
    s = stream_ptr(torch)
    need = tm.tm_op_linear_dgrad_scratch_bytes(BF16, T, N, K)
    assert need == 8 * T * K * 4                 # eight parts of 512
    assert tm.tm_op_linear_dgrad_scratch_bytes(BF16, 2048, 4608, 12288) == 0   # enough tiles: no split
    scratch = torch.empty(need, dtype=torch.uint8, device="cuda")
    new = lambda: torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    a, b, c, d = new(), new(), new(), new()
    tm.tm_op_linear_dgrad_ws(BF16, T, N, K, dyd, wd, a, scratch, need, s)
    tm.tm_op_linear_dgrad_ws(BF16, T, N, K, dyd, wd, b, scratch, need, s)
    tm.tm_op_linear_dgrad_ws(BF16, T, N, K, dyd, wd, c, None, 0, s)
    tm.tm_op_linear_dgrad(BF16, T, N, K, dyd, wd, d, s)
    torch.cuda.synchronize()
    ref = dy.astype(np.float64) @ w.astype(np.float64)
    assert rel_err(to_host(a), ref) <= TOL_BF16 and rel_err(to_host(d), ref) <= TOL_BF16
    assert torch.equal(a, b) and torch.equal(c, d)


def test_input_gradient_with_split_reduction_on_large_tiles(env):
    """Same, at a shape whose parts fill the chip with 256 x 192 tiles (the kernel with loader waves writes the fp32
    partial results): ragged in both output dimensions, eight parts of 512."""
    torch, tm = env
    T, N, K = 1000, 4096, 1096                   # 4 x 6 large tiles, eight parts: 192 blocks
    rng = np.random.default_rng(22)
    dy, w = rand(rng, (T, N), 0.1, BF16), rand(rng, (N, K), 0.05, BF16)
    dyd, wd = to_dev(torch, dy, BF16), to_dev(torch, w, BF16)
    s = stream_ptr(torch)
    need = tm.tm_op_linear_dgrad_scratch_bytes(BF16, T, N, K)
    assert need == 8 * T * K * 4
    scratch = torch.empty(need, dtype=torch.uint8, device="cuda")
    new = lambda: torch.full((T, K), float("nan"), dtype=torch.bfloat16, device="cuda")
    a, b, c = new(), new(), new()
    tm.tm_op_linear_dgrad_ws(BF16, T, N, K, dyd, wd, a, scratch, need, s)
    scratch.fill_(255)                           # stale partial results must not matter
    tm.tm_op_linear_dgrad_ws(BF16, T, N, K, dyd, wd, b, scratch, need, s)
    tm.tm_op_linear_dgrad(BF16, T, N, K, dyd, wd, c, s)
    torch.cuda.synchronize()
    ref = dy.astype(np.float64) @ w.astype(np.float64)
    assert rel_err(to_host(a), ref) <= TOL_BF16 and rel_err(to_host(c), ref) <= TOL_BF16
    assert torch.equal(a, b)


def test_gradient_overwrite_mode_ignores_old_contents(env):
    torch, tm = env
    rng = np.random.default_rng(4)
    T, N, K = 300, 264, 192
    x, dy = rand(rng, (T, K), 1.0, BF16), rand(rng, (T, N), 0.1, BF16)
    xd, dyd = to_dev(torch, x, BF16), to_dev(torch, dy, BF16)
    s = stream_ptr(torch)
    dw = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    tm.tm_op_linear_wgrad(BF16, T, N, K, dyd, xd, dw, 0, s)
    assert rel_err(to_host(dw), dy.astype(np.float64).T @ x.astype(np.float64)) <= 1e-5
    db = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
    scratch = torch.empty(tm.tm_op_reduce_scratch_bytes(T, 2 * N), dtype=torch.uint8, device="cuda")
    tm.tm_op_bias_grad(BF16, T, N, dyd, db, scratch, 0, s)
    assert rel_err(to_host(db), dy.astype(np.float64).sum(axis=0)) <= 1e-5
    # fp32 stage dtype goes through the plain-ALU kernel
    dwf = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    tm.tm_op_linear_wgrad(FP32, T, N, K, dyd.float(), xd.float(), dwf, 0, s)
    assert rel_err(to_host(dwf), dy.astype(np.float64).T @ x.astype(np.float64)) <= 1e-5


def test_linear_results_are_bit_reproducible(env):
    torch, tm = env
    rng = np.random.default_rng(3)
    T, N, K = 384, 264, 320
    x, w, dy = rand(rng, (T, K), 1.0, BF16), rand(rng, (N, K), 0.05, BF16), rand(rng, (T, N), 0.1, BF16)
    xd, wd, dyd = (to_dev(torch, a, BF16) for a in (x, w, dy))
    outs = []
    for _ in range(2):
        y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
        dw = torch.zeros((N, K), dtype=torch.float32, device="cuda")
        tm.tm_op_linear_fwd(BF16, T, N, K, xd, wd, None, None, y, stream_ptr(torch))
        tm.tm_op_linear_wgrad(BF16, T, N, K, dyd, xd, dw, 1, stream_ptr(torch))
        outs.append((y, dw))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


# ------------------------------------------------------------------ bias gradient
@pytest.mark.parametrize("dtype,T,N", [(BF16, 300, 264), (BF16, 5, 8), (FP32, 131, 72), (BF16, 2048, 1536)])
def test_bias_grad(env, dtype, T, N):
    torch, tm = env
    rng = np.random.default_rng(11)
    dy = rand(rng, (T, N), 0.1, dtype)
    g0 = rng.standard_normal(N).astype(np.float32)
    db = f32_dev(torch, g0)
    scratch = torch.empty(tm.tm_op_reduce_scratch_bytes(T, N), dtype=torch.uint8, device="cuda")
    tm.tm_op_bias_grad(dtype, T, N, to_dev(torch, dy, dtype), db, scratch, 1, stream_ptr(torch))
    assert rel_err(to_host(db), g0 + dy.astype(np.float64).sum(axis=0)) <= 1e-5


# ------------------------------------------------------------------ norms
@pytest.mark.parametrize("dtype,kind,T,h", [
    (BF16, so.NORM_LAYERNORM, 37, 264), (BF16, so.NORM_RMSNORM, 37, 264), (BF16, so.NORM_LAYERNORM, 9, 12288),
    (BF16, so.NORM_RMSNORM, 300, 8192), (FP32, so.NORM_LAYERNORM, 37, 256), (FP32, so.NORM_RMSNORM, 1, 8),
    (BF16, so.NORM_LAYERNORM, 600, 16384)])
def test_norm_fwd_bwd(env, dtype, kind, T, h):
    torch, tm = env
    print(f"norm dtype={dtype} kind={kind} T={T} h={h}", flush=True)
    rng = np.random.default_rng(h + T)
    x = rand(rng, (T, h), 1.5, dtype, mean=0.3)
    gain, off = rand(rng, (h,), 0.1, dtype, mean=1.0), rand(rng, (h,), 0.1, dtype)
    dout, dres = rand(rng, (T, h), 0.1, dtype), rand(rng, (T, h), 0.1, dtype)
    eps = 1e-5
    td = torch_dtype(torch, dtype)
    s = stream_ptr(torch)
    xd, gd, od = to_dev(torch, x, dtype), to_dev(torch, gain, dtype), to_dev(torch, off, dtype)
    out = torch.empty((T, h), dtype=td, device="cuda")
    mean = torch.zeros(T, dtype=torch.float32, device="cuda")
    rstd = torch.zeros(T, dtype=torch.float32, device="cuda")
    ln = kind == so.NORM_LAYERNORM
    tm.tm_op_norm_fwd(dtype, kind, T, h, eps, xd, gd, od if ln else None, out, mean if ln else None, rstd, s)
    ref, xhat, r = so.norm_fwd(x, gain.astype(np.float64), off.astype(np.float64) if ln else None, kind, eps)
    assert rel_err(to_host(out), ref) <= tol_of(dtype)
    assert rel_err(to_host(rstd), r[:, 0]) <= 1e-5
    if ln:
        assert np.abs(to_host(mean) - x.astype(np.float64).mean(axis=1)).max() <= 1e-5

    dx = torch.empty((T, h), dtype=td, device="cuda")
    g0, o0 = rng.standard_normal(h).astype(np.float32), rng.standard_normal(h).astype(np.float32)
    dgain, doff = f32_dev(torch, g0), f32_dev(torch, o0)
    scratch = torch.empty(tm.tm_op_reduce_scratch_bytes(T, 3 * h), dtype=torch.uint8, device="cuda")
    tm.tm_op_norm_bwd(dtype, kind, T, h, to_dev(torch, dout, dtype), xd, mean if ln else None, rstd, gd,
                      to_dev(torch, dres, dtype), dx, dgain, doff if ln else None, scratch, 1, s)
    rdx, rdg, rdo = so.norm_bwd(dout, xhat, r, gain.astype(np.float64), kind)
    assert rel_err(to_host(dx), rdx + dres) <= tol_of(dtype)
    assert rel_err(to_host(dgain), g0 + rdg) <= 1e-4
    if ln:
        assert rel_err(to_host(doff), o0 + rdo) <= 1e-4
    # without a residual gradient, and storing instead of adding the gain / offset gradients
    tm.tm_op_norm_bwd(dtype, kind, T, h, to_dev(torch, dout, dtype), xd, mean if ln else None, rstd, gd, None, dx,
                      dgain, doff if ln else None, scratch, 0, s)
    assert rel_err(to_host(dx), rdx) <= tol_of(dtype)
    assert rel_err(to_host(dgain), rdg) <= 1e-4
    if ln:
        assert rel_err(to_host(doff), rdo) <= 1e-4
    # the variant that also returns the column sums of dx (a bias gradient without another pass): same dx, same
    # gain / offset gradients bit for bit, and the sums of the values as stored
    dx2 = torch.empty_like(dx)
    dg2, do2 = torch.empty_like(dgain), torch.empty_like(doff)
    c0 = rng.standard_normal(h).astype(np.float32)
    csum = f32_dev(torch, c0)
    tm.tm_op_norm_bwd(dtype, kind, T, h, to_dev(torch, dout, dtype), xd, mean if ln else None, rstd, gd,
                      to_dev(torch, dres, dtype), dx, dgain, doff if ln else None, scratch, 0, s)
    tm.tm_op_norm_bwd_colsum(dtype, kind, T, h, to_dev(torch, dout, dtype), xd, mean if ln else None, rstd, gd,
                             to_dev(torch, dres, dtype), dx2, dg2, do2 if ln else None, csum, scratch, 0, s)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx2) and torch.equal(dgain, dg2) and (not ln or torch.equal(doff, do2))
    assert rel_err(to_host(csum), to_host(dx2).sum(axis=0)) <= 1e-5
    tm.tm_op_norm_bwd_colsum(dtype, kind, T, h, to_dev(torch, dout, dtype), xd, mean if ln else None, rstd, gd,
                             to_dev(torch, dres, dtype), dx2, dg2, do2 if ln else None, csum, scratch, 1, s)
    assert rel_err(to_host(csum), 2.0 * to_host(dx2).sum(axis=0)) <= 1e-5
    assert rel_err(to_host(csum), 2.0 * (rdx + dres).sum(axis=0)) <= tol_of(dtype)


# ------------------------------------------------------------------ activations
@pytest.mark.parametrize("dtype", [BF16, FP32])
@pytest.mark.parametrize("act", [so.ACT_GELU_TANH, so.ACT_GELU_ERF, so.ACT_SWIGLU])
def test_activation_fwd_bwd(env, dtype, act):
    torch, tm = env
    rng = np.random.default_rng(act + 5)
    T, f = 77, 136
    width = 2 * f if act == so.ACT_SWIGLU else f
    u = rand(rng, (T, width), 2.0, dtype)
    dg = rand(rng, (T, f), 0.1, dtype)
    td = torch_dtype(torch, dtype)
    s = stream_ptr(torch)
    ud = to_dev(torch, u, dtype)
    g = torch.empty((T, f), dtype=td, device="cuda")
    du = torch.empty((T, width), dtype=td, device="cuda")
    tm.tm_op_act_fwd(dtype, act, T, f, ud, g, s)
    tm.tm_op_act_bwd(dtype, act, T, f, to_dev(torch, dg, dtype), ud, du, s)
    u64, dg64 = u.astype(np.float64), dg.astype(np.float64)
    if act == so.ACT_SWIGLU:
        ref = so.swiglu_fwd(u64[:, :f], u64[:, f:])
        rdu = np.concatenate(so.swiglu_bwd(dg64, u64[:, :f], u64[:, f:]), axis=1)
    else:
        ref, rdu = so.gelu_fwd(u64, act), so.gelu_bwd(dg64, u64, act)
    tol = TOL_BF16 if dtype == BF16 else 1e-5
    assert rel_err(to_host(g), ref) <= tol
    assert rel_err(to_host(du), rdu) <= tol


# ------------------------------------------------------------------ rotary
@pytest.mark.parametrize("dtype,seq,batch,heads,d", [(BF16, 33, 2, 3, 128), (FP32, 17, 1, 2, 8), (BF16, 4100, 1, 1, 64)])
def test_rotary_forward_and_inverse(env, dtype, seq, batch, heads, d):
    torch, tm = env
    rng = np.random.default_rng(seq)
    width = (heads + 2) * d        # two trailing heads (the V part) must stay untouched
    z = rand(rng, (seq, batch, width), 1.0, dtype)
    buf = to_dev(torch, z, dtype)
    tm.tm_op_rotary(dtype, seq, batch, heads, d, width, 10000.0, 0, buf, stream_ptr(torch))
    ang = so.rotary_angles(seq, d, 10000.0)
    z64 = z.astype(np.float64)
    ref = z64.copy()
    ref[..., :heads * d] = so.rotary_apply(z64[..., :heads * d].reshape(seq, batch, heads, d), ang).reshape(seq, batch, -1)
    got = to_host(buf)
    assert rel_err(got, ref) <= (TOL_BF16 if dtype == BF16 else 1e-5)
    assert (got[..., heads * d:] == z64[..., heads * d:]).all()
    tm.tm_op_rotary(dtype, seq, batch, heads, d, width, 10000.0, 1, buf, stream_ptr(torch))
    assert rel_err(to_host(buf), z64) <= (TOL_BF16 if dtype == BF16 else 1e-5)


# ------------------------------------------------------------------ attention
ATTN_SHAPES = [
    # dtype, seq, batch, nq, nkv, d
    (BF16, 300, 2, 4, 2, 128),   # MFMA path, grouped heads, ragged: 2 query blocks + tail, 5 key tiles
    (BF16, 128, 1, 2, 2, 128),   # exactly one block
    (BF16, 1, 1, 1, 1, 128),     # a single position: ctx = v
    (BF16, 200, 1, 2, 1, 64),    # MFMA path with head size 64
    (BF16, 70, 2, 2, 1, 32),     # plain-ALU path in bf16
    (FP32, 128, 2, 4, 4, 64),    # the tiny preset's attention
    (FP32, 45, 1, 4, 2, 16),
]


@pytest.mark.parametrize("dtype,seq,batch,nq,nkv,d", ATTN_SHAPES)
def test_attention_fwd_bwd(env, dtype, seq, batch, nq, nkv, d):
    torch, tm = env
    print(f"attention dtype={dtype} seq={seq} batch={batch} nq={nq} nkv={nkv} d={d}", flush=True)
    rng = np.random.default_rng(seq * 3 + d)
    A, W = nq * d, (nq + 2 * nkv) * d
    qkv = rand(rng, (seq, batch, W), 1.0, dtype)
    dctx = rand(rng, (seq, batch, A), 0.1, dtype)
    td = torch_dtype(torch, dtype)
    s = stream_ptr(torch)
    qd = to_dev(torch, qkv, dtype)
    ctx = torch.empty((seq, batch, A), dtype=td, device="cuda")
    lse = torch.zeros((batch, nq, seq), dtype=torch.float32, device="cuda")
    tm.tm_op_attn_fwd(dtype, seq, batch, nq, nkv, d, qd, ctx, lse, s)
    q64 = qkv.astype(np.float64)
    q = q64[..., :A].reshape(seq, batch, nq, d)
    k = q64[..., A:A + nkv * d].reshape(seq, batch, nkv, d)
    v = q64[..., A + nkv * d:].reshape(seq, batch, nkv, d)
    ref = so.attention_fwd(q, k, v)
    tol = tol_of(dtype)
    assert rel_err(to_host(ctx), ref.reshape(seq, batch, A)) <= tol
    # log-sum-exp of the scaled scores, from the definition
    for n in range(batch):
        for g in (0, nq - 1):
            sc = q[:, n, g] @ k[:, n, g // (nq // nkv)].T / math.sqrt(d)
            sc = np.where(np.tril(np.ones((seq, seq), bool)), sc, -np.inf)
            mx = sc.max(axis=1)
            ref_lse = mx + np.log(np.exp(sc - mx[:, None]).sum(axis=1))
            assert np.abs(to_host(lse[n, g]) - ref_lse).max() <= (1e-3 if dtype == BF16 else 1e-4)

    dqkv = torch.zeros((seq, batch, W), dtype=td, device="cuda")
    dvec = torch.empty(tm.tm_op_attn_bwd_scratch_bytes(dtype, seq, batch, nq, nkv, d), dtype=torch.uint8, device="cuda")
    tm.tm_op_attn_bwd(dtype, seq, batch, nq, nkv, d, qd, ctx, to_dev(torch, dctx, dtype), lse, dvec, dqkv, s)
    dq, dk, dv = so.attention_bwd(dctx.astype(np.float64).reshape(seq, batch, nq, d), q, k, v)
    got = to_host(dqkv)
    assert rel_err(got[..., :A], dq.reshape(seq, batch, A)) <= tol
    assert rel_err(got[..., A:A + nkv * d], dk.reshape(seq, batch, -1)) <= tol
    assert rel_err(got[..., A + nkv * d:], dv.reshape(seq, batch, -1)) <= tol


@pytest.mark.parametrize("split", ["0", "1"], ids=["four_wave_blocks", "eight_wave_split_key_tiles"])
@pytest.mark.parametrize("seq,batch,nq,nkv", [(700, 1, 3, 3), (300, 2, 4, 2), (64, 1, 1, 1), (1, 1, 2, 1), (129, 1, 2, 2)],
                         ids=["ragged_11_key_tiles", "grouped_heads", "one_key_tile", "one_position", "one_row_past_a_block"])
def test_attention_block_forms(env, monkeypatch, split, seq, batch, nq, nkv):
    """The head-size-128 forward kernel comes in two block forms, chosen by the grid size (TM_ATTN_SPLIT forces one): four
    waves walking all key tiles of their query rows, and eight waves where two waves share the query rows and take the
    even and the odd key tiles (their softmax states merged at the end).  Both against the checker (and the backward
    pass from each one's log-sum-exp);
    with one key tile the odd side has nothing to do and must contribute nothing."""
    torch, tm = env
    monkeypatch.setenv("TM_ATTN_SPLIT", split)
    d, dtype = 128, BF16
    print(f"attention block form split={split} seq={seq} batch={batch} nq={nq} nkv={nkv}", flush=True)
    rng = np.random.default_rng(seq * 7 + nq)
    A, W = nq * d, (nq + 2 * nkv) * d
    qkv = rand(rng, (seq, batch, W), 1.0, dtype)
    dctx = rand(rng, (seq, batch, A), 0.1, dtype)
    s = stream_ptr(torch)
    qd = to_dev(torch, qkv, dtype)
    ctx = torch.empty((seq, batch, A), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((batch, nq, seq), dtype=torch.float32, device="cuda")
    tm.tm_op_attn_fwd(dtype, seq, batch, nq, nkv, d, qd, ctx, lse, s)
    q64 = qkv.astype(np.float64)
    q = q64[..., :A].reshape(seq, batch, nq, d)
    k = q64[..., A:A + nkv * d].reshape(seq, batch, nkv, d)
    v = q64[..., A + nkv * d:].reshape(seq, batch, nkv, d)
    tol = tol_of(dtype)
    assert rel_err(to_host(ctx), so.attention_fwd(q, k, v).reshape(seq, batch, A)) <= tol
    sc = q[:, 0, nq - 1] @ k[:, 0, (nq - 1) // (nq // nkv)].T / math.sqrt(d)
    sc = np.where(np.tril(np.ones((seq, seq), bool)), sc, -np.inf)
    mx = sc.max(axis=1)
    assert np.abs(to_host(lse[0, nq - 1]) - (mx + np.log(np.exp(sc - mx[:, None]).sum(axis=1)))).max() <= 1e-3
    dqkv = torch.zeros((seq, batch, W), dtype=torch.bfloat16, device="cuda")
    scratch = torch.empty(tm.tm_op_attn_bwd_scratch_bytes(dtype, seq, batch, nq, nkv, d), dtype=torch.uint8, device="cuda")
    tm.tm_op_attn_bwd(dtype, seq, batch, nq, nkv, d, qd, ctx, to_dev(torch, dctx, dtype), lse, scratch, dqkv, s)
    dq, dk, dv = so.attention_bwd(dctx.astype(np.float64).reshape(seq, batch, nq, d), q, k, v)
    got = to_host(dqkv)
    assert rel_err(got[..., :A], dq.reshape(seq, batch, A)) <= tol
    assert rel_err(got[..., A:A + nkv * d], dk.reshape(seq, batch, -1)) <= tol
    assert rel_err(got[..., A + nkv * d:], dv.reshape(seq, batch, -1)) <= tol


@pytest.mark.parametrize("both", ["0", "1"], ids=["two_launches", "one_launch"])
@pytest.mark.parametrize("seq,batch,nq,nkv", [(700, 1, 3, 3), (300, 2, 4, 2), (64, 1, 1, 1), (1, 1, 2, 1), (129, 1, 2, 2),
                                               (193, 1, 2, 1)],
                         ids=["ragged_11_key_tiles", "grouped_heads", "one_key_tile", "one_position", "one_row_past_a_block",
                              "one_row_past_a_key_tile"])
def test_attention_backward_launch_forms(env, monkeypatch, both, seq, batch, nq, nkv):
    """The head-size-128 backward pass runs as two launches (dQ blocks, then dK/dV blocks) or, for grids that leave
    compute units idle, as one launch that holds both kinds of blocks (TM_ATTN_BWD_BOTH forces one).  Each form against
    the checker; nothing may be written past the tensor's last row."""
    torch, tm = env
    monkeypatch.setenv("TM_ATTN_BWD_BOTH", both)
    d, dtype = 128, BF16
    print(f"attention backward form both={both} seq={seq} batch={batch} nq={nq} nkv={nkv}", flush=True)
    rng = np.random.default_rng(seq * 11 + nq)
    A, W = nq * d, (nq + 2 * nkv) * d
    qkv = rand(rng, (seq, batch, W), 1.0, dtype)
    dctx = rand(rng, (seq, batch, A), 0.1, dtype)
    s = stream_ptr(torch)
    qd = to_dev(torch, qkv, dtype)
    ctx = torch.empty((seq, batch, A), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((batch, nq, seq), dtype=torch.float32, device="cuda")
    tm.tm_op_attn_fwd(dtype, seq, batch, nq, nkv, d, qd, ctx, lse, s)
    q64 = qkv.astype(np.float64)
    q = q64[..., :A].reshape(seq, batch, nq, d)
    k = q64[..., A:A + nkv * d].reshape(seq, batch, nkv, d)
    v = q64[..., A + nkv * d:].reshape(seq, batch, nkv, d)
    tol = tol_of(dtype)
    guard = 64                                      # rows after the tensor: nothing may be written there
    dqkv = torch.full((seq + guard, batch, W), float("nan"), dtype=torch.bfloat16, device="cuda")
    scratch = torch.empty(tm.tm_op_attn_bwd_scratch_bytes(dtype, seq, batch, nq, nkv, d), dtype=torch.uint8, device="cuda")
    tm.tm_op_attn_bwd(dtype, seq, batch, nq, nkv, d, qd, ctx, to_dev(torch, dctx, dtype), lse, scratch, dqkv[:seq], s)
    torch.cuda.synchronize()
    assert torch.isnan(dqkv[seq:]).all()
    dq, dk, dv = so.attention_bwd(dctx.astype(np.float64).reshape(seq, batch, nq, d), q, k, v)
    got = to_host(dqkv[:seq])
    assert np.isfinite(got).all()
    assert rel_err(got[..., :A], dq.reshape(seq, batch, A)) <= tol
    assert rel_err(got[..., A:A + nkv * d], dk.reshape(seq, batch, -1)) <= tol
    assert rel_err(got[..., A + nkv * d:], dv.reshape(seq, batch, -1)) <= tol


@pytest.mark.parametrize("seq,batch,nq,nkv", [(700, 1, 3, 3), (300, 2, 4, 2), (257, 1, 2, 1), (1, 1, 1, 1)],
                         ids=["ragged_3_blocks", "grouped_heads", "one_row_past_a_block", "one_position"])
def test_attention_blocks_of_256_query_rows(env, monkeypatch, seq, batch, nq, nkv):
    """Long sequences run the forward and the dQ walk in blocks of 256 query rows (eight waves sharing every staged key /
    value tile).  TM_ATTN_WIDE=1 forces that form on small shapes (with the other forms switched off): against the
    checker, and nothing written past the last row."""
    torch, tm = env
    monkeypatch.setenv("TM_ATTN_WIDE", "1")
    monkeypatch.setenv("TM_ATTN_SPLIT", "0")
    monkeypatch.setenv("TM_ATTN_BWD_BOTH", "0")
    d, dtype = 128, BF16
    print(f"attention 256-row blocks seq={seq} batch={batch} nq={nq} nkv={nkv}", flush=True)
    rng = np.random.default_rng(seq * 13 + nq)
    A, W = nq * d, (nq + 2 * nkv) * d
    qkv = rand(rng, (seq, batch, W), 1.0, dtype)
    dctx = rand(rng, (seq, batch, A), 0.1, dtype)
    s = stream_ptr(torch)
    qd = to_dev(torch, qkv, dtype)
    guard = 64
    ctx = torch.full((seq + guard, batch, A), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((batch, nq, seq), dtype=torch.float32, device="cuda")
    tm.tm_op_attn_fwd(dtype, seq, batch, nq, nkv, d, qd, ctx[:seq], lse, s)
    q64 = qkv.astype(np.float64)
    q = q64[..., :A].reshape(seq, batch, nq, d)
    k = q64[..., A:A + nkv * d].reshape(seq, batch, nkv, d)
    v = q64[..., A + nkv * d:].reshape(seq, batch, nkv, d)
    tol = tol_of(dtype)
    torch.cuda.synchronize()
    assert torch.isnan(ctx[seq:]).all()
    assert rel_err(to_host(ctx[:seq]), so.attention_fwd(q, k, v).reshape(seq, batch, A)) <= tol
    dqkv = torch.full((seq + guard, batch, W), float("nan"), dtype=torch.bfloat16, device="cuda")
    scratch = torch.empty(tm.tm_op_attn_bwd_scratch_bytes(dtype, seq, batch, nq, nkv, d), dtype=torch.uint8, device="cuda")
    tm.tm_op_attn_bwd(dtype, seq, batch, nq, nkv, d, qd, ctx[:seq], to_dev(torch, dctx, dtype), lse, scratch, dqkv[:seq], s)
    torch.cuda.synchronize()
    assert torch.isnan(dqkv[seq:]).all()
    dq, dk, dv = so.attention_bwd(dctx.astype(np.float64).reshape(seq, batch, nq, d), q, k, v)
    got = to_host(dqkv[:seq])
    assert np.isfinite(got).all()
    assert rel_err(got[..., :A], dq.reshape(seq, batch, A)) <= tol
    assert rel_err(got[..., A:A + nkv * d], dk.reshape(seq, batch, -1)) <= tol
    assert rel_err(got[..., A + nkv * d:], dv.reshape(seq, batch, -1)) <= tol


def test_attention_is_bit_reproducible(env):
    torch, tm = env
    rng = np.random.default_rng(8)
    seq, batch, nq, nkv, d = 260, 1, 4, 1, 128
    A, W = nq * d, (nq + 2 * nkv) * d
    qd = to_dev(torch, rand(rng, (seq, batch, W), 1.0, BF16), BF16)
    dc = to_dev(torch, rand(rng, (seq, batch, A), 0.1, BF16), BF16)
    outs = []
    for _ in range(2):
        ctx = torch.empty((seq, batch, A), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((batch, nq, seq), dtype=torch.float32, device="cuda")
        dqkv = torch.empty((seq, batch, W), dtype=torch.bfloat16, device="cuda")
        dvec = torch.empty(tm.tm_op_attn_bwd_scratch_bytes(BF16, seq, batch, nq, nkv, d), dtype=torch.uint8, device="cuda")
        tm.tm_op_attn_fwd(BF16, seq, batch, nq, nkv, d, qd, ctx, lse, stream_ptr(torch))
        tm.tm_op_attn_bwd(BF16, seq, batch, nq, nkv, d, qd, ctx, dc, lse, dvec, dqkv, stream_ptr(torch))
        outs.append((ctx, lse, dqkv))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# ------------------------------------------------------------------ Adam
@pytest.mark.parametrize("n,lowp,zero,step,wd,gs", [(1000003, True, False, 1, 0.0, 1.0), (4096, False, True, 7, 0.01, 0.5),
                                                    (5, True, True, 2, 0.0, 1.0), (8, True, False, 1000, 0.1, 1.0)])
def test_adam_flat_matches_fp64_definition(env, n, lowp, zero, step, wd, gs):
    torch, tm = env
    p, g, m, v = si.make_adam_state(n, seed=step)
    pd, gd, md, vd = (f32_dev(torch, a) for a in (p, g, m, v))
    lo = torch.zeros(n, dtype=torch.bfloat16, device="cuda") if lowp else None
    hp = tm.make_hparams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=wd, grad_scale=gs, zero_grads=zero)
    tm.tm_adam_step_flat(n, pd, gd, md, vd, lo, hp, step, stream_ptr(torch))
    rp, rm, rv = so.adam_step(p, g, m, v, step, 1e-3, 0.9, 0.999, 1e-8, wd, gs)
    assert rel_err(to_host(pd), rp) <= TOL_ADAM
    assert rel_err(to_host(md), rm) <= TOL_ADAM
    assert rel_err(to_host(vd), rv) <= TOL_ADAM
    if lowp:
        # the bf16 copy is the nearest-even rounding of the fp32 weight the kernel itself stored
        want = so.bf16_round_nearest_even(pd.cpu().numpy())
        got = lo.view(torch.int16).cpu().numpy().view(np.uint16)
        assert (got == want).all()
    if zero:
        assert float(gd.abs().max()) == 0.0
    else:
        assert torch.equal(gd.cpu(), torch.from_numpy(g))


def test_adam_first_step_closed_form(env):
    torch, tm = env
    n = 10000
    p, g, _, _ = si.make_adam_state(n)
    pd, gd = f32_dev(torch, p), f32_dev(torch, g)
    md, vd = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    tm.tm_adam_step_flat(n, pd, gd, md, vd, None, tm.make_hparams(), 1, stream_ptr(torch))
    ref = p.astype(np.float64) - 1e-3 * g.astype(np.float64) / (np.abs(g.astype(np.float64)) + 1e-8)
    assert rel_err(to_host(pd), ref) <= TOL_ADAM


# ------------------------------------------------------------------ argument errors
@pytest.mark.parametrize("n", [1, 7, 4096, 4097, 1_000_003])
def test_sum_of_squares(env, n):
    torch, tm = env
    rng = np.random.default_rng(n)
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    gd = f32_dev(torch, g)
    scratch = torch.empty(tm.tm_sq_sum_scratch_bytes(n), dtype=torch.uint8, device="cuda")
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    tm.tm_sq_sum(n, gd, scratch, out, stream_ptr(torch))
    tm.tm_sq_sum(n, gd, scratch, out[1:], stream_ptr(torch))
    torch.cuda.synchronize()
    ref = so.grad_sq_sum(g)
    assert abs(float(out[0]) - ref) <= 1e-6 * ref
    assert float(out[0]) == float(out[1])               # fixed summation order


def test_bad_arguments_are_reported_not_launched(env):
    torch, tm = env
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    with pytest.raises(tm.TmError) as e:
        tm.tm_op_linear_fwd(BF16, 4, 12, 8, t, t, None, None, t, 0)       # N not a multiple of 8
    assert e.value.code == tm.TM_ESIZE
    with pytest.raises(tm.TmError) as e:
        tm.tm_op_linear_fwd(BF16, 4, 8, 8, None, t, None, None, t, 0)
    assert e.value.code == tm.TM_EINVAL
    with pytest.raises(tm.TmError) as e:
        tm.tm_adam_step_flat(8, t, t, t, t, None, tm.make_hparams(), 0, 0)  # step < 1
    assert e.value.code == tm.TM_EINVAL
    with pytest.raises(tm.TmError) as e:
        tm.tm_op_attn_fwd(BF16, 16, 1, 3, 2, 64, t, t, t, 0)               # heads not divisible
    assert e.value.code == tm.TM_ESIZE
    with pytest.raises(tm.TmError) as e:
        tm.tm_op_norm_fwd(BF16, 0, 4, 32768, 1e-5, t, t, t, t, t, t, 0)    # row too wide
    assert e.value.code == tm.TM_ESIZE
