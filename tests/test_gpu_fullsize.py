"""Parity at the full shard sizes of the presets, in the launch configuration the benchmark
times.  Products and attention are checked on sampled output rows the CPU checker evaluates one by
one from the definition; stage iterations at full width and reduced depth are compared in full."""
import math
import os
import time

import numpy as np
import pytest

import synth_inputs as si
from oracle import stage_oracle as so
from tests.gpu_util import (TOL_ADAM, TOL_BF16, f32_dev, rand, rel_err, require_gpu, stream_ptr, to_dev, to_host)
from tests.test_gpu_stage import run_and_compare

pytestmark = pytest.mark.gpu
BF16 = si.DTYPE_BF16


@pytest.fixture(scope="module")
def env():
    torch = require_gpu()
    import paper_2412_12636_amd as tm
    return torch, tm


def _bf16_normal(torch, shape, std, seed):
    """Device-side draw (too large for a host generator in test time), values on the bf16 grid."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return (torch.empty(shape, dtype=torch.float32, device="cuda").normal_(0, std, generator=g)).to(torch.bfloat16)


LINEAR_FULL = [("gpt175b qkv", 2048, 4608, 12288), ("gpt175b out", 2048, 12288, 1536),
               ("gpt175b fc1", 2048, 6144, 12288), ("gpt175b fc2", 2048, 12288, 6144),
               ("llama70b fc1", 4096, 7168, 8192), ("longctx qkv", 16384, 1280, 8192)]


@pytest.mark.parametrize("name,T,N,K", LINEAR_FULL, ids=[c[0].replace(" ", "_") for c in LINEAR_FULL])
def test_linear_full_size_sampled_rows(env, name, T, N, K):
    torch, tm = env
    print(f"full-size linear {name}: T={T} N={N} K={K}", flush=True)
    x, w = _bf16_normal(torch, (T, K), 1.0, 1), _bf16_normal(torch, (N, K), 0.02, 2)
    dy, bias = _bf16_normal(torch, (T, N), 0.01, 3), _bf16_normal(torch, (N,), 0.02, 4)
    s = stream_ptr(torch)
    y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    dw = torch.zeros((N, K), dtype=torch.float32, device="cuda")
    res = x[:, :N].contiguous() if K >= N else None
    tm.tm_op_linear_fwd(BF16, T, N, K, x, w, bias, res, y, s)
    tm.tm_op_linear_dgrad(BF16, T, N, K, dy, w, dx, s)
    tm.tm_op_linear_wgrad(BF16, T, N, K, dy, x, dw, 1, s)
    torch.cuda.synchronize()
    rng = np.random.default_rng(T + N)
    rows_t = sorted(set([0, 127, 128, T - 1] + rng.integers(0, T, 12).tolist()))
    rows_n = sorted(set([0, 191, 192, N - 1] + rng.integers(0, N, 12).tolist()))
    xh, wh, dyh, bh = to_host(x), to_host(w), to_host(dy), to_host(bias)
    ref = xh[rows_t] @ wh.T + bh
    if K >= N:
        ref = ref + xh[rows_t][:, :N]
    assert rel_err(to_host(y[rows_t]), ref) <= TOL_BF16
    assert rel_err(to_host(dx[rows_t]), dyh[rows_t] @ wh) <= TOL_BF16
    assert rel_err(to_host(dw[rows_n]), dyh[:, rows_n].T @ xh) <= 1e-5
    assert bool(torch.isfinite(y.float()).all()) and bool(torch.isfinite(dx.float()).all())


def test_attention_long_context_sampled_rows(env):
    """seq 16384, 8 query heads on 1 kv head: forward rows, dQ rows and dK/dV rows from the definition."""
    torch, tm = env
    seq, batch, nq, nkv, d = 16384, 1, 8, 1, 128
    A, W = nq * d, (nq + 2 * nkv) * d
    qkv = _bf16_normal(torch, (seq, batch, W), 1.0, 11)
    dctx = _bf16_normal(torch, (seq, batch, A), 0.01, 12)
    s = stream_ptr(torch)
    ctx = torch.empty((seq, batch, A), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((batch, nq, seq), dtype=torch.float32, device="cuda")
    dvec = torch.empty(tm.tm_op_attn_bwd_scratch_bytes(BF16, seq, batch, nq, nkv, d), dtype=torch.uint8, device="cuda")
    dqkv = torch.empty_like(qkv)
    tm.tm_op_attn_fwd(BF16, seq, batch, nq, nkv, d, qkv, ctx, lse, s)
    tm.tm_op_attn_bwd(BF16, seq, batch, nq, nkv, d, qkv, ctx, dctx, lse, dvec, dqkv, s)
    torch.cuda.synchronize()
    print("long-context attention launched; evaluating the definition on the host", flush=True)
    q64 = to_host(qkv)[:, 0]
    q, k, v = q64[:, :A].reshape(seq, nq, d), q64[:, A:A + d], q64[:, A + d:]
    dc = to_host(dctx)[:, 0].reshape(seq, nq, d)
    scale = 1.0 / math.sqrt(d)
    rows = [0, 1, 63, 64, 127, 128, 4097, 9999, seq - 1]
    got_ctx, got_lse, got_d = to_host(ctx)[:, 0].reshape(seq, nq, d), to_host(lse)[0], to_host(dqkv)[:, 0]
    # forward rows and dQ rows
    for i in rows:
        sc = (q[i] @ k[:i + 1].T) * scale                    # [nq, i+1]
        mx = sc.max(axis=1, keepdims=True)
        e = np.exp(sc - mx)
        z = e.sum(axis=1, keepdims=True)
        p = e / z
        ref = p @ v[:i + 1]
        assert rel_err(got_ctx[i], ref) <= TOL_BF16, i
        assert np.abs(got_lse[:, i] - (mx + np.log(z))[:, 0]).max() <= 1e-3
        dp = dc[i] @ v[:i + 1].T
        ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
        assert rel_err(got_d[i, :A].reshape(nq, d), ds @ k[:i + 1] * scale) <= TOL_BF16, i
    # dK/dV rows need the softmax denominators of every later query row: blocked pass per head
    t0 = time.time()
    lse_ref = np.empty((nq, seq))
    dsum = (dc * 1.0)                                         # D_i = dctx_i . ctx_i, from the definition of ctx
    Dv = np.empty((nq, seq))
    blk = 2048
    for g in range(nq):
        for i0 in range(0, seq, blk):
            sc = (q[i0:i0 + blk, g] @ k[:i0 + blk].T) * scale
            sc = np.where(np.arange(i0, i0 + blk)[:, None] >= np.arange(i0 + blk)[None, :], sc, -np.inf)
            mx = sc.max(axis=1, keepdims=True)
            e = np.exp(sc - mx)
            z = e.sum(axis=1, keepdims=True)
            lse_ref[g, i0:i0 + blk] = (mx + np.log(z))[:, 0]
            Dv[g, i0:i0 + blk] = (((e / z) @ v[:i0 + blk]) * dsum[i0:i0 + blk, g]).sum(axis=1)
        print(f"  head {g}: reference statistics after {time.time() - t0:.0f} s", flush=True)
    for j in [0, 64, 8191, seq - 130, seq - 1]:
        dk, dv = np.zeros(d), np.zeros(d)
        for g in range(nq):
            pj = np.exp((q[j:, g] @ k[j]) * scale - lse_ref[g, j:])          # column j of P, rows j..
            dpj = dc[j:, g] @ v[j]
            dsj = pj * (dpj - Dv[g, j:])
            dv += pj @ dc[j:, g]
            dk += dsj @ q[j:, g] * scale
        assert rel_err(got_d[j, A:A + d], dk) <= TOL_BF16, j
        assert rel_err(got_d[j, A + d:], dv) <= TOL_BF16, j
    assert bool(torch.isfinite(dqkv.float()).all())


def test_adam_sweep_sampled_elements(env):
    """1.2e9 parameters: every element is independent, so a sample pins the whole launch."""
    torch, tm = env
    n = si.ADAM_SWEEP_ELEMS
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    p = torch.empty(n, device="cuda").normal_(0, 0.02, generator=g)
    gr = torch.empty(n, device="cuda").normal_(0, 1e-3, generator=g)
    m = torch.empty(n, device="cuda").normal_(0, 1e-4, generator=g)
    v = torch.empty(n, device="cuda").normal_(0, 1e-3, generator=g).square_().mul_(1e-3)
    idx = torch.from_numpy(np.unique(np.r_[0, 1, 2, 3, n - 4, n - 3, n - 2, n - 1,
                                          np.random.default_rng(0).integers(0, n, 200000)])).cuda()
    before = [to_host(t[idx]) for t in (p, gr, m, v)]
    lo = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    tm.tm_adam_step_flat(n, p, gr, m, v, lo, tm.make_hparams(weight_decay=0.01, zero_grads=1), 3, stream_ptr(torch))
    torch.cuda.synchronize()
    rp, rm, rv = so.adam_step(*before, 3, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1.0)
    assert rel_err(to_host(p[idx]), rp) <= TOL_ADAM
    assert rel_err(to_host(m[idx]), rm) <= TOL_ADAM and rel_err(to_host(v[idx]), rv) <= TOL_ADAM
    want = so.bf16_round_nearest_even(p[idx].cpu().numpy())
    assert (lo[idx].view(torch.int16).cpu().numpy().view(np.uint16) == want).all()
    assert float(gr.abs().max()) == 0.0


# Max-norm tolerance of a whole stage at full width against the fp64 checker, by depth.  One layer meets the stated
# 2e-2 (measured 1.5e-2 / 1.3e-2 / 1.4e-2 at the three widths).  From the second layer on a layer inherits the
# rounding of the layers around it, and at these widths it amplifies what it inherits (tests/test_depth_reading.py:
# a perturbation of one bf16 rounding on a layer's input moves the gradients that pass through the softmax 2.4 to
# 3.3 times as much, the residual stream 1.75 times), so the distance to an fp64 reference grows with depth although
# every layer on its own, given the same inputs, stays within 2e-2 (the chain test below).  Measured worst tensor:
# 175B shard 3.6e-2 at 2 layers, 6.5e-2 at 4, 1.08e-1 at 12 (y: 1.3e-2, 1.8e-2, 2.2e-2); Llama-70B shard 2.7e-2 at 2.
# The table holds the asserted bounds (measured values with a margin of about a quarter); y keeps 2e-2 up to 4 layers.
DEPTH_TOL = {("gpt175b", 1): 2e-2, ("llama70b", 1): 2e-2, ("longctx", 1): 2e-2,
             ("gpt175b", 2): 4.5e-2, ("llama70b", 2): 3.5e-2, ("gpt175b", 12): 1.4e-1}
Y_TOL_DEEP = 3e-2          # stage output at 12 layers (measured 2.2e-2)
# (one layer at the 175B width is held to 2e-2 by the chain test below, layers 0 and 11)
STAGE_CASES = [("llama70b", 1), ("longctx", 1), ("gpt175b", 2), ("llama70b", 2)]


@pytest.mark.parametrize("preset,layers", STAGE_CASES, ids=[f"{p}_L{l}" for p, l in STAGE_CASES])
def test_stage_full_width_reduced_depth(env, progress, preset, layers):
    """Whole-stage parity at the full width of the three large presets: one layer to the stated tolerance (the
    16384-token shard included), two layers to the depth table above; every tensor's error and elementwise pass
    rate are reported."""
    torch, tm = env
    cfg = si.PRESETS[preset].replace(n_layers=layers)
    progress(f"stage parity {preset} at full width, {layers} layer(s)")
    tol = DEPTH_TOL[(preset, layers)]
    report = {}
    run_and_compare(torch, tm, cfg, progress=progress, tol=lambda name: TOL_BF16 if name == "y" else tol, report=report)
    worst = sorted(report.items(), key=lambda kv: -kv[1][0])[:4]
    progress("  " + "; ".join(f"{k} err {e:.2e} pass {r:.4f}" for k, (e, r) in worst))


@pytest.mark.skipif(os.environ.get("TM_TEST_FULL_DEPTH") != "1",
                    reason="five minutes of fp64 checker time and about 110 GB of host memory: run with TM_TEST_FULL_DEPTH=1")
def test_gpt175b_full_depth_against_checker(env, progress):
    """The benchmark's workload, all 12 layers, against the fp64 checker run over the whole stage (measured: worst
    tensor 1.08e-1 on a QKV weight gradient, y 2.2e-2, dx 8.2e-2; see the depth table)."""
    torch, tm = env
    cfg = si.PRESETS["gpt175b"]
    report = {}
    run_and_compare(torch, tm, cfg, progress=progress, adam=False, report=report,
                    tol=lambda name: Y_TOL_DEEP if name == "y" else DEPTH_TOL[("gpt175b", 12)])
    worst = sorted(report.items(), key=lambda kv: -kv[1][0])[:6]
    progress("  " + "; ".join(f"{k} err {e:.2e} pass {r:.4f}" for k, (e, r) in worst))


def test_gpt175b_full_depth_equals_chained_layers_and_layers_match_checker(env):
    """The benchmark's workload: 12 layers at the 175B-shard width.

    Against the fp64 checker run over the whole stage the distance grows with depth (depth table above; the full
    run is test_gpt175b_full_depth_against_checker).  What the stated 2e-2 can and does hold is every layer on its
    own; the full-depth run is therefore also pinned in two steps that together say so:
      1. the 12-layer call is BIT-IDENTICAL to twelve 1-layer calls chained through their own
         outputs (same kernels, same order: pins sequencing, stash and gradient offsets);
      2. individual layers of that chain (first and last) match the checker to 2e-2 when the checker
         is given the same layer input and output gradient."""
    torch, tm = env
    cfg = si.PRESETS["gpt175b"]
    one = cfg.replace(n_layers=1)
    n, n1 = tm.tm_stage_param_count(cfg), tm.tm_stage_param_count(one)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(si.BASE_SEED)
    master = torch.empty(n, dtype=torch.float32, device="cuda")
    for lo in range(0, n, 1 << 28):
        master[lo:lo + (1 << 28)].normal_(0.0, 0.02, generator=gen)
    for name, off, shape in tm.tm_stage_param_layout(cfg):
        if name.endswith("_gain"):
            master[off:off + shape[0]] += 1.0
    params = master.to(torch.bfloat16)
    master.copy_(params)
    grads = torch.zeros(n, dtype=torch.float32, device="cuda")
    m, v = torch.zeros(8, device="cuda"), torch.zeros(8, device="cuda")   # Adam is not called here
    shape = (cfg.seq, cfg.micro_batch, cfg.hidden)
    x = torch.empty(shape, device="cuda").normal_(0, 1, generator=gen).to(torch.bfloat16)
    dy = torch.empty(shape, device="cuda").normal_(0, 1e-2, generator=gen).to(torch.bfloat16)
    s = stream_ptr(torch)
    print("full-depth stage: forward and backward of 12 layers", flush=True)
    ws = torch.empty(tm.tm_stage_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    h = tm.tm_stage_init(cfg, params, master, grads, master, master, ws)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    tm.tm_stage_fwd(h, x, y, s)
    tm.tm_stage_bwd(h, dy, dx, s)
    torch.cuda.synchronize()
    tm.tm_stage_destroy(h)
    assert bool(torch.isfinite(y.float()).all()) and bool(torch.isfinite(dx.float()).all())

    print("chain of 1-layer stages", flush=True)
    grads1 = torch.zeros(n, dtype=torch.float32, device="cuda")
    ws1 = torch.empty(tm.tm_stage_workspace_bytes(one), dtype=torch.uint8, device="cuda")
    xs = [x]
    for l in range(cfg.n_layers):
        hl = tm.tm_stage_init(one, params[l * n1:], master[l * n1:], grads1[l * n1:], master, master, ws1)
        out = torch.empty_like(x)
        tm.tm_stage_fwd(hl, xs[-1], out, s)
        xs.append(out)
        tm.tm_stage_destroy(hl)
    assert torch.equal(xs[-1], y)
    dys = {cfg.n_layers: dy}
    for l in reversed(range(cfg.n_layers)):
        hl = tm.tm_stage_init(one, params[l * n1:], master[l * n1:], grads1[l * n1:], master, master, ws1)
        tmp, out = torch.empty_like(x), torch.empty_like(x)
        tm.tm_stage_fwd(hl, xs[l], tmp, s)
        tm.tm_stage_bwd(hl, dys[l + 1], out, s)
        dys[l] = out
        tm.tm_stage_destroy(hl)
    torch.cuda.synchronize()
    assert torch.equal(dys[0], dx)
    # Below the top layer the FC2 bias gradient (column sums of the layer's output gradient) comes out of the first
    # norm's backward pass of the layer above, in a 1-layer stage out of the column-sum kernel: the same stored
    # values added in another order.  Those entries agree to fp32 summation accuracy, everything else bit for bit.
    for name, off, shape in tm.tm_stage_param_layout(cfg):
        if name.endswith(".b_fc2") and not name.startswith(f"layer{cfg.n_layers - 1}."):
            a, b = grads1[off:off + shape[0]].double(), grads[off:off + shape[0]].double()
            assert float((a - b).abs().max() / b.abs().max()) <= 1e-5, name
            grads1[off:off + shape[0]] = grads[off:off + shape[0]]       # checked: leave the rest to the exact comparison
    assert torch.equal(grads1, grads)

    for l in (0, cfg.n_layers - 1):
        print(f"layer {l} of the chain against the checker", flush=True)
        flat = params[l * n1:(l + 1) * n1].float().cpu().numpy()
        layer = si.split_flat(one, flat)[0]
        t0 = time.time()
        ry, st = so.layer_fwd(one, layer, to_host(xs[l]))
        print(f"  checker forward done at {time.time() - t0:.0f} s", flush=True)
        rdx, rg = so.layer_bwd(one, layer, st, to_host(dys[l + 1]))
        print(f"  checker backward done at {time.time() - t0:.0f} s", flush=True)
        assert rel_err(to_host(xs[l + 1]), ry) <= TOL_BF16
        assert rel_err(to_host(dys[l]), rdx) <= TOL_BF16
        gl = grads[l * n1:(l + 1) * n1].cpu().numpy().astype(np.float64)
        off = 0
        for name, shp in si.layer_inventory(one):
            k = int(np.prod(shp))
            e = rel_err(gl[off:off + k], rg[name].reshape(-1))
            assert e <= TOL_BF16, (l, name, e)
            off += k


def test_gpt175b_benchmark_configuration_equals_the_three_calls(env):
    """The launch configuration the benchmark times (12 layers at the 175B-shard width, measured tile
    configurations, transient gradients, tm_stage_fwd + tm_stage_bwd_adam with every weight matrix updated in
    the epilogue of its weight-gradient product) against the plain sequence tm_stage_fwd, tm_stage_bwd,
    tm_adam_step on a second copy of the same state: outputs, input gradients, master weights, both moments
    and the bf16 weights bit for bit over two iterations (the second forward pass reads updated weights and
    the moments are no longer zero).  The plain sequence is the one the other tests hold against the checker."""
    torch, tm = env
    cfg = si.PRESETS["gpt175b"]
    n = tm.tm_stage_param_count(cfg)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(si.BASE_SEED + 7)
    master0 = torch.empty(n, dtype=torch.float32, device="cuda")
    for lo in range(0, n, 1 << 28):
        master0[lo:lo + (1 << 28)].normal_(0.0, 0.02, generator=gen)
    for name, off, shape in tm.tm_stage_param_layout(cfg):
        if name.endswith("_gain"):
            master0[off:off + shape[0]] += 1.0
    params0 = master0.to(torch.bfloat16)
    master0.copy_(params0)
    shape = (cfg.seq, cfg.micro_batch, cfg.hidden)
    x = torch.empty(shape, device="cuda").normal_(0, 1, generator=gen).to(torch.bfloat16)
    dy = torch.empty(shape, device="cuda").normal_(0, 1e-2, generator=gen).to(torch.bfloat16)
    s = stream_ptr(torch)

    def state():
        st = {"params": params0.clone(), "master": master0.clone(), "grads": torch.zeros(n, device="cuda"),
              "m": torch.zeros(n, device="cuda"), "v": torch.zeros(n, device="cuda"),
              "ws": torch.empty(tm.tm_stage_workspace_bytes(cfg), dtype=torch.uint8, device="cuda"),
              "y": torch.empty_like(x), "dx": torch.empty_like(x)}
        st["h"] = tm.tm_stage_init(cfg, st["params"], st["master"], st["grads"], st["m"], st["v"], st["ws"])
        return st

    print("benchmark configuration at full size: building two states", flush=True)
    a, b = state(), state()
    del master0, params0
    tm.tm_stage_grad_mode(b["h"], tm.TM_GRAD_TRANSIENT)
    tm.tm_stage_tune(b["h"], s)
    hp_plain = tm.make_hparams(**si.ADAM_DEFAULTS, zero_grads=1)
    hp = tm.make_hparams(**si.ADAM_DEFAULTS)
    for step in (1, 2):
        print(f"  iteration {step}: three calls, then forward + backward-with-update", flush=True)
        tm.tm_stage_fwd(a["h"], x, a["y"], s)
        tm.tm_stage_bwd(a["h"], dy, a["dx"], s)
        tm.tm_adam_step(a["h"], hp_plain, step, s)
        tm.tm_stage_fwd(b["h"], x, b["y"], s)
        tm.tm_stage_bwd_adam(b["h"], dy, b["dx"], hp, step, s)
        torch.cuda.synchronize()
        for name in ("y", "dx", "master", "m", "v", "params"):
            assert torch.equal(a[name], b[name]), (step, name)
        assert bool(torch.isfinite(a["y"].float()).all())
    # the update moved the weights, and by no more than the step size allows (|delta| <= lr per step for Adam)
    moved = (a["master"][:1 << 24] - a["params"][:1 << 24].float()).abs().max()
    assert float(moved) <= 2 ** -8 * float(a["master"][:1 << 24].abs().max())   # bf16 copy = rounded master
    tm.tm_stage_destroy(a["h"])
    tm.tm_stage_destroy(b["h"])
