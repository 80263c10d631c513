"""First- and last-stage layers on the GPU (through the C ABI) against the fp64 checker."""
from __future__ import annotations

import numpy as np
import pytest

import synth_inputs as si
from oracle import roles_oracle as ro
from oracle import stage_oracle as so
from tests.gpu_util import TOL_BF16, TOL_FP32, f32_dev, rand, rel_err, require_gpu, stream_ptr, to_dev, to_host, torch_dtype

pytestmark = pytest.mark.gpu
BF16, FP32 = si.DTYPE_BF16, si.DTYPE_FP32


@pytest.fixture(scope="module")
def env():
    torch = require_gpu()
    import paper_2412_12636_amd as tm
    return torch, tm


def _tokens(rng, lo, hi, shape):
    return rng.integers(lo, hi, size=shape).astype(np.int32)


@pytest.mark.parametrize("dtype,seq,batch,h,v_local,with_pos", [
    (BF16, 70, 3, 264, 40, True),       # ragged everything, ids below / inside / above the shard
    (BF16, 1100, 1, 512, 96, False),    # more tokens than one scan window of the backward kernel
    (FP32, 33, 2, 72, 24, True),
])
def test_embedding_forward_and_backward(env, dtype, seq, batch, h, v_local, with_pos):
    torch, tm = env
    print(f"embedding dtype={dtype} seq={seq} batch={batch} h={h} v_local={v_local} pos={with_pos}", flush=True)
    rng = np.random.default_rng(seq + h)
    v0, n_pos = 100, seq + 5
    tokens = _tokens(rng, v0 - v_local // 2, v0 + v_local + v_local // 2, (seq, batch))
    w = rand(rng, (v_local, h), 0.02, dtype)
    pos = rand(rng, (n_pos, h), 0.02, dtype) if with_pos else None
    dx0 = rand(rng, (seq, batch, h), 0.1, dtype)
    td = torch_dtype(torch, dtype)
    s = stream_ptr(torch)
    tok_d = torch.from_numpy(tokens.reshape(-1)).cuda()
    x0 = torch.empty((seq, batch, h), dtype=td, device="cuda")
    tm.tm_op_embed_fwd(dtype, seq, batch, h, v_local, v0, tok_d, to_dev(torch, w, dtype),
                       to_dev(torch, pos, dtype) if with_pos else None, x0, s)
    ref = ro.embedding_fwd(tokens, w, v0, pos)
    assert rel_err(to_host(x0), ref) <= (TOL_BF16 if dtype == BF16 else 1e-6)

    g0 = rng.standard_normal((v_local, h)).astype(np.float32)
    p0 = rng.standard_normal((n_pos, h)).astype(np.float32)
    rdw, rdp = ro.embedding_bwd(dx0, tokens, v_local, v0, n_pos if with_pos else 0)
    for accumulate in (1, 0):
        dw, dp = f32_dev(torch, g0), f32_dev(torch, p0)
        tm.tm_op_embed_bwd(dtype, seq, batch, h, v_local, v0, tok_d, to_dev(torch, dx0, dtype), dw,
                           dp if with_pos else None, n_pos, accumulate, s)
        torch.cuda.synchronize()
        base = g0.astype(np.float64) if accumulate else 0.0
        assert rel_err(to_host(dw), base + rdw) <= 1e-5          # fp32 sums of exactly representable inputs
        if with_pos:
            assert rel_err(to_host(dp), (p0.astype(np.float64) if accumulate else 0.0) + rdp) <= 1e-5
    dw2 = torch.empty((v_local, h), dtype=torch.float32, device="cuda")
    tm.tm_op_embed_bwd(dtype, seq, batch, h, v_local, v0, tok_d, to_dev(torch, dx0, dtype), dw2, None, 0, 0, s)
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw)                                  # reproducible


@pytest.mark.parametrize("dtype,T,v_local", [(BF16, 37, 264), (BF16, 5, 2056), (FP32, 19, 72)])
def test_cross_entropy_over_the_shard(env, dtype, T, v_local):
    torch, tm = env
    print(f"xent dtype={dtype} T={T} v_local={v_local}", flush=True)
    rng = np.random.default_rng(T)
    v0 = 16
    logits = rand(rng, (T, v_local), 2.0, dtype)
    targets = _tokens(rng, 0, v0 + v_local + 16, (T,))
    targets[0], targets[1] = v0, v0 + v_local - 1                # both ends of the shard
    s = stream_ptr(torch)
    ld = to_dev(torch, logits, dtype)
    loss_t = torch.empty(T, dtype=torch.float32, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    tm.tm_op_xent(dtype, T, v_local, v0, ld, torch.from_numpy(targets).cuda(), 3.0, loss_t, loss, s)
    torch.cuda.synchronize()
    ref_t, probs = ro.xent_fwd(logits, targets, v0)
    assert rel_err(to_host(loss_t), ref_t) <= 1e-5
    assert abs(float(loss) - ref_t.mean()) <= 1e-5 * abs(ref_t.mean())
    ref_d = ro.xent_bwd(probs, targets, v0, np.full(T, 3.0 / T))
    assert rel_err(to_host(ld), ref_d) <= (TOL_BF16 if dtype == BF16 else 1e-5)


HEAD_CASES = [
    (BF16, so.NORM_LAYERNORM, 60, 2, 256, 200),     # K = 200 in the input-gradient product: staged kernel
    (BF16, so.NORM_RMSNORM, 130, 1, 512, 320),      # pipelined kernels
    (FP32, so.NORM_LAYERNORM, 24, 2, 64, 40),
]


@pytest.mark.parametrize("dtype,norm,seq,batch,h,v_local", HEAD_CASES)
def test_last_stage_forward_and_backward(env, dtype, norm, seq, batch, h, v_local):
    torch, tm = env
    print(f"head dtype={dtype} norm={norm} seq={seq} batch={batch} h={h} v_local={v_local}", flush=True)
    rng = np.random.default_rng(seq * 3 + h)
    T, v0 = seq * batch, 1000
    y = rand(rng, (seq, batch, h), 1.0, dtype)
    gain = rand(rng, (h,), 0.02, dtype, mean=1.0)
    offset = rand(rng, (h,), 0.02, dtype) if norm == so.NORM_LAYERNORM else None
    w = rand(rng, (v_local, h), 0.05, dtype)
    targets = _tokens(rng, v0 - 10, v0 + v_local + 10, (seq, batch))
    td = torch_dtype(torch, dtype)
    s = stream_ptr(torch)
    ws = torch.empty(tm.tm_head_workspace_bytes(dtype, seq, batch, h, v_local), dtype=torch.uint8, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    dy = torch.empty((seq, batch, h), dtype=td, device="cuda")
    dgain = torch.zeros(h, dtype=torch.float32, device="cuda")
    doffset = torch.zeros(h, dtype=torch.float32, device="cuda")
    dw = torch.zeros((v_local, h), dtype=torch.float32, device="cuda")
    args = (dtype, norm, 1e-5, seq, batch, h, v_local, v0, to_dev(torch, y, dtype), torch.from_numpy(targets.reshape(-1)).cuda(),
            to_dev(torch, gain, dtype), to_dev(torch, offset, dtype) if offset is not None else None, to_dev(torch, w, dtype), 1.0,
            ws, loss, dy, dgain, doffset if offset is not None else None, dw)
    tm.tm_head_fwd_bwd(*args, accumulate=0, stream=s)
    torch.cuda.synchronize()
    rloss, st = ro.head_fwd(norm, 1e-5, y, gain, offset, w, targets, v0)
    rdy, rdgain, rdoffset, rdw = ro.head_bwd(norm, st, gain, w, targets, v0)
    tol = TOL_BF16 if dtype == BF16 else TOL_FP32
    assert abs(float(loss) - rloss) <= tol * abs(rloss)
    assert rel_err(to_host(dy), rdy) <= tol
    assert rel_err(to_host(dw), rdw) <= tol
    assert rel_err(to_host(dgain), rdgain) <= tol
    if offset is not None:
        assert rel_err(to_host(doffset), rdoffset) <= tol
    # accumulate mode adds the same amounts once more
    first = dw.clone()
    tm.tm_head_fwd_bwd(*args, accumulate=1, stream=s)
    torch.cuda.synchronize()
    assert rel_err(to_host(dw), 2.0 * to_host(first)) <= 1e-6
    # a workspace one byte short is refused
    with pytest.raises(tm.TmError) as e:
        tm.tm_head_fwd_bwd(*args, accumulate=0, stream=s, workspace_bytes=ws.numel() - 1)
    assert e.value.code == tm.TM_ESIZE


def test_last_stage_at_the_175b_shard_width(env):
    """hidden 12288, 2048 tokens, 6400 vocabulary rows per rank (51200 / 8): loss, sampled rows of dy and of
    dW, and the norm-gain gradient, against the checker (which forms the full logits once)."""
    torch, tm = env
    seq, batch, h, v_local, v0 = 2048, 1, 12288, 6400, 12800
    T = seq * batch
    print(f"last stage full width: T={T} h={h} v_local={v_local}", flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)

    def draw(shape, std, mean=0.0):
        return torch.empty(shape, dtype=torch.float32, device="cuda").normal_(mean, std, generator=gen).to(torch.bfloat16)

    y, gain, offset, w = draw((seq, batch, h), 1.0), draw((h,), 0.02, 1.0), draw((h,), 0.02), draw((v_local, h), 0.02)
    targets = torch.randint(0, 51200, (T,), generator=gen, device="cuda", dtype=torch.int32)
    targets[:T // 2] = torch.randint(v0, v0 + v_local, (T // 2,), generator=gen, device="cuda", dtype=torch.int32)
    s = stream_ptr(torch)
    ws = torch.empty(tm.tm_head_workspace_bytes(BF16, seq, batch, h, v_local), dtype=torch.uint8, device="cuda")
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    dy = torch.empty_like(y)
    dgain = torch.empty(h, dtype=torch.float32, device="cuda")
    doffset = torch.empty(h, dtype=torch.float32, device="cuda")
    dw = torch.empty((v_local, h), dtype=torch.float32, device="cuda")
    tm.tm_head_fwd_bwd(BF16, so.NORM_LAYERNORM, 1e-5, seq, batch, h, v_local, v0, y, targets, gain, offset, w, 1.0, ws, loss,
                       dy, dgain, doffset, dw, accumulate=0, stream=s)
    torch.cuda.synchronize()
    yh, gh, oh, wh = (to_host(t) for t in (y, gain, offset, w))
    th = targets.cpu().numpy().reshape(seq, batch)
    rloss, st = ro.head_fwd(so.NORM_LAYERNORM, 1e-5, yh, gh, oh, wh, th, v0)
    rdy, rdgain, rdoffset, rdw = ro.head_bwd(so.NORM_LAYERNORM, st, gh, wh, th, v0)
    print(f"  loss gpu {float(loss):.6f} checker {rloss:.6f}", flush=True)
    assert abs(float(loss) - rloss) <= 2e-3 * abs(rloss)
    rows = np.random.default_rng(5).choice(T, 48, replace=False)
    vrows = np.random.default_rng(6).choice(v_local, 48, replace=False)
    dyh = to_host(dy).reshape(T, h)
    assert rel_err(dyh[rows], rdy.reshape(T, h)[rows]) <= TOL_BF16
    assert rel_err(to_host(dw[torch.from_numpy(vrows).cuda()]), rdw[vrows]) <= TOL_BF16
    assert rel_err(to_host(dgain), rdgain) <= TOL_BF16 and rel_err(to_host(doffset), rdoffset) <= TOL_BF16
    assert bool(torch.isfinite(dy.float()).all()) and bool(torch.isfinite(dw).all())


def test_embedding_at_the_175b_shard_width(env):
    torch, tm = env
    seq, batch, h, v_local, v0 = 2048, 1, 12288, 6400, 12800
    gen = torch.Generator(device="cuda")
    gen.manual_seed(78)
    w = torch.empty((v_local, h), dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=gen).to(torch.bfloat16)
    pos = torch.empty((seq, h), dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=gen).to(torch.bfloat16)
    dx0 = torch.empty((seq, batch, h), dtype=torch.float32, device="cuda").normal_(0, 0.01, generator=gen).to(torch.bfloat16)
    tokens = torch.randint(v0 - 100, v0 + v_local + 100, (seq * batch,), generator=gen, device="cuda", dtype=torch.int32)
    tokens[:64] = v0 + 5                                   # one row collects many tokens
    s = stream_ptr(torch)
    x0 = torch.empty((seq, batch, h), dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((v_local, h), dtype=torch.float32, device="cuda")
    dp = torch.empty((seq, h), dtype=torch.float32, device="cuda")
    tm.tm_op_embed_fwd(BF16, seq, batch, h, v_local, v0, tokens, w, pos, x0, s)
    tm.tm_op_embed_bwd(BF16, seq, batch, h, v_local, v0, tokens, dx0, dw, dp, seq, 0, s)
    torch.cuda.synchronize()
    th = tokens.cpu().numpy().reshape(seq, batch)
    assert rel_err(to_host(x0), ro.embedding_fwd(th, to_host(w), v0, to_host(pos))) <= TOL_BF16
    rdw, rdp = ro.embedding_bwd(to_host(dx0), th, v_local, v0, seq)
    assert rel_err(to_host(dw), rdw) <= 1e-5 and rel_err(to_host(dp), rdp) <= 1e-5
