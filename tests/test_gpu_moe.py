"""The mixture-of-experts MLP shard through the C ABI against the fp64 CPU checker: routing decisions exactly,
everything else within the storage tolerance; small shapes with drops, ragged sizes and several expert-parallel
groupings, then the 5.12T-shaped shard on sampled outputs."""
import time

import numpy as np
import pytest

import synth_inputs as si
from oracle import moe_oracle as mo
from oracle import stage_oracle as so
from tests.gpu_util import TOL_BF16, TOL_FP32, f32_dev, rel_err, require_gpu, stream_ptr, to_dev, to_host

pytestmark = pytest.mark.gpu
BF16, FP32 = si.DTYPE_BF16, si.DTYPE_FP32


@pytest.fixture(scope="module")
def env():
    torch = require_gpu()
    import paper_2412_12636_amd as tm
    return torch, tm


def cap(T, k, E, factor):
    return si.moe_capacity(T, k, E, factor)


CASES = {
    "fp32_groups": si.MoeConfig(150, 64, 96, 8, 2, 2, cap(150, 2, 8, 1.0), dtype=FP32),
    "bf16_drops": si.MoeConfig(300, 256, 512, 8, 4, 2, cap(300, 2, 8, 1.0)),
    "bf16_one_local_expert": si.MoeConfig(260, 128, 256, 16, 16, 2, cap(260, 2, 16, 1.25)),
    "bf16_top1_all_local": si.MoeConfig(200, 128, 192, 4, 1, 1, cap(200, 1, 4, 0.75)),
    "bf16_top3_erf_nobias": si.MoeConfig(129, 192, 320, 6, 3, 3, cap(129, 3, 6, 1.0), act=si.ACT_GELU_ERF, has_bias=0),
    "bf16_roomy": si.MoeConfig(70, 64, 64, 4, 2, 2, 70),
    # the degenerate ends: one token; buffers of one row (almost everything dropped); 64 experts with top-8 (both maxima);
    # a single expert (gate 1, the router gets no gradient)
    "one_token": si.MoeConfig(1, 64, 64, 4, 2, 2, 1),
    "capacity_one": si.MoeConfig(40, 64, 72, 4, 1, 2, 1),
    "max_experts_max_k": si.MoeConfig(90, 64, 64, 64, 8, 8, si.moe_capacity(90, 8, 64, 1.0)),
    "single_expert": si.MoeConfig(33, 72, 136, 1, 1, 1, 20),
}


def flat_of(cfg, tm, p):
    layout = tm.tm_moe_param_layout(cfg)
    inv = si.moe_inventory(cfg)
    assert [n for n, _, _ in layout] == [n for n, _ in inv]
    flat = np.empty(tm.tm_moe_param_count(cfg), dtype=np.float32)
    for (name, off, shape), (_, ishape) in zip(layout, inv):
        assert shape == (ishape[0], ishape[1] if len(ishape) == 2 else 1) and off % 8 == 0
        flat[off:off + p[name].size] = p[name].reshape(-1)
    return flat, layout


def library_row(cfg, oracle_row):
    """Row numbering of the checker (expert * capacity + position) -> the library's buffer order."""
    e, pos = oracle_row // cfg.capacity, oracle_row % cfg.capacity
    el = cfg.n_experts // cfg.ep
    return np.where(oracle_row < 0, -1, ((e % el) * cfg.ep + e // el) * cfg.capacity + pos)


def read_ws(torch, tm, cfg, ws, region, dtype):
    off, nbytes = tm.tm_moe_workspace_offset(cfg, region)
    return ws[off:off + nbytes].view(dtype).cpu().numpy()


@pytest.mark.parametrize("name", list(CASES))
def test_moe_shard_matches_checker(env, name):
    torch, tm = env
    cfg = CASES[name]
    print(f"moe parity {name}: {cfg}", flush=True)
    tol = TOL_BF16 if cfg.dtype == BF16 else TOL_FP32
    p = si.make_moe_params(cfg, router_std=0.05)
    c, dout = si.make_moe_io(cfg)
    E, ep, k, C = cfg.n_experts, cfg.ep, cfg.top_k, cfg.capacity
    rout, st = mo.moe_fwd(c, p, E, ep, k, C, cfg.act)
    rdc, rgr = mo.moe_bwd(dout, p, st, E, ep, k, C, cfg.act)
    margin = mo.min_decision_margin(st["logits"], min(k, E - 1)) if E > 1 else float("inf")
    dropped = int((st["row"] < 0).sum())
    print(f"  decision margin {margin:.2e}, dropped assignments {dropped} of {cfg.tokens * k}", flush=True)
    assert margin > 2e-5, "the seeded inputs must keep the routing decision away from ties"
    if name in ("bf16_drops", "fp32_groups", "bf16_top1_all_local"):
        assert dropped > 0
    if name == "bf16_roomy":
        assert dropped == 0

    flat, layout = flat_of(cfg, tm, p)
    td = torch.bfloat16 if cfg.dtype == BF16 else torch.float32
    pd, cd, dd = to_dev(torch, flat, cfg.dtype), to_dev(torch, c, cfg.dtype), to_dev(torch, dout, cfg.dtype)
    ws = torch.empty(tm.tm_moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    out = torch.empty((cfg.tokens, cfg.hidden), dtype=td, device="cuda")
    dc = torch.empty_like(out)
    grads = torch.full((flat.size,), 7.0, dtype=torch.float32, device="cuda")      # overwritten, not added to
    s = stream_ptr(torch)
    tm.tm_moe_fwd(cfg, pd, cd, out, ws, s)
    torch.cuda.synchronize()
    # routing: integers exactly, fp32 quantities tightly
    assert rel_err(read_ws(torch, tm, cfg, ws, tm.TM_MOE_WS_LOGITS, torch.float32), st["logits"].reshape(-1)) <= 1e-5
    assert (read_ws(torch, tm, cfg, ws, tm.TM_MOE_WS_TOP_IDX, torch.int32).reshape(-1, k) == st["idx"]).all()
    assert rel_err(read_ws(torch, tm, cfg, ws, tm.TM_MOE_WS_GATES, torch.float32), st["gates"].reshape(-1)) <= 1e-5
    assert (read_ws(torch, tm, cfg, ws, tm.TM_MOE_WS_SLOT_ROW, torch.int32).reshape(-1, k) == library_row(cfg, st["row"])).all()
    e_out = rel_err(to_host(out), rout)
    tm.tm_moe_bwd(cfg, pd, cd, dd, dc, grads, 0, ws, s)
    torch.cuda.synchronize()
    errs = {"out": e_out, "dc": rel_err(to_host(dc), rdc)}
    g = grads.cpu().numpy().astype(np.float64)
    for nm, off, shape in layout:
        errs[nm] = rel_err(g[off:off + shape[0] * shape[1]], rgr[nm].reshape(-1))
    worst = max(errs, key=errs.get)
    print(f"  worst {worst}: {errs[worst]:.3e}  out {errs['out']:.3e}  dc {errs['dc']:.3e}", flush=True)
    assert errs[worst] <= tol, errs
    # dropped tokens: exactly zero where every assignment was dropped
    all_dropped = (st["row"] < 0).all(axis=1)
    if all_dropped.any():
        assert (to_host(out)[all_dropped] == 0).all()
    # a second pass adds the same gradients; a repeat of everything gives the same bits
    out1, dc1, g1 = out.clone(), dc.clone(), grads.clone()
    tm.tm_moe_bwd(cfg, pd, cd, dd, dc, grads, 1, ws, s)
    torch.cuda.synchronize()
    assert rel_err(to_host(grads), 2.0 * g) <= 1e-6
    tm.tm_moe_fwd(cfg, pd, cd, out, ws, s)
    tm.tm_moe_bwd(cfg, pd, cd, dd, dc, grads, 0, ws, s)
    torch.cuda.synchronize()
    assert torch.equal(out, out1) and torch.equal(dc, dc1) and torch.equal(grads, g1)


def test_moe_argument_errors(env):
    torch, tm = env
    cfg = CASES["bf16_roomy"]
    for bad, code in ((cfg.replace(hidden=100), tm.TM_ESIZE), (cfg.replace(n_experts=65), tm.TM_ESIZE),
                      (cfg.replace(ep=3), tm.TM_ESIZE), (cfg.replace(top_k=5), tm.TM_ESIZE), (cfg.replace(capacity=0), tm.TM_EINVAL),
                      (cfg.replace(act=si.ACT_SWIGLU), tm.TM_EINVAL), (cfg.replace(dtype=5), tm.TM_EINVAL)):
        with pytest.raises(tm.TmError) as e:
            tm.tm_moe_workspace_bytes(bad)
        assert e.value.code == code
    n = tm.tm_moe_param_count(cfg)
    pd = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    x = torch.zeros((cfg.tokens, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(tm.tm_moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    with pytest.raises(tm.TmError) as e:
        tm.tm_moe_fwd(cfg, pd, x, x, ws, stream_ptr(torch), workspace_bytes=ws.numel() - 1)
    assert e.value.code == tm.TM_ESIZE
    with pytest.raises(tm.TmError) as e:
        tm.tm_moe_fwd(cfg, pd, None, x, ws, stream_ptr(torch))
    assert e.value.code == tm.TM_EINVAL
    with pytest.raises(tm.TmError) as e:
        tm.tm_moe_workspace_offset(cfg, 9)
    assert e.value.code == tm.TM_EINVAL


def test_moe_at_the_5t_shard_shape_on_sampled_outputs(env):
    """2048 tokens, hidden 20480, one local expert of width 10240, 16 experts, top-2: the checker routes every token,
    forms the expert's first product once (the only large CPU product), and computes sampled rows / columns of
    every output from their definitions."""
    torch, tm = env
    cfg = si.MOE_PRESETS["moe5t"]
    T, h, f, E, ep, k, C = cfg.tokens, cfg.hidden, cfg.ffn, cfg.n_experts, cfg.ep, cfg.top_k, cfg.capacity
    print(f"moe full size: {cfg}", flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(si.BASE_SEED + 3)
    n = tm.tm_moe_param_count(cfg)
    pd = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=gen).to(torch.bfloat16)
    cd = torch.empty((T, h), dtype=torch.float32, device="cuda").normal_(0, 1, generator=gen).to(torch.bfloat16)
    dd = torch.empty((T, h), dtype=torch.float32, device="cuda").normal_(0, 1e-2, generator=gen).to(torch.bfloat16)
    ws = torch.empty(tm.tm_moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    out, dc = torch.empty_like(cd), torch.empty_like(cd)
    grads = torch.empty(n, dtype=torch.float32, device="cuda")
    s = stream_ptr(torch)
    tm.tm_moe_fwd(cfg, pd, cd, out, ws, s)
    tm.tm_moe_bwd(cfg, pd, cd, dd, dc, grads, 0, ws, s)
    torch.cuda.synchronize()
    t0 = time.time()
    layout = {nm: (off, shape) for nm, off, shape in tm.tm_moe_param_layout(cfg)}
    host = lambda nm: to_host(pd[layout[nm][0]:layout[nm][0] + layout[nm][1][0] * layout[nm][1][1]]).reshape(layout[nm][1])
    c, dout = to_host(cd), to_host(dd)
    wr, w1, w2 = host("w_router"), host("w_fc1.0"), host("w_fc2.0")
    b1, b2 = host("b_fc1.0").reshape(-1), host("b_fc2.0").reshape(-1)
    logits, idx, gates = mo.router(c, wr, k)
    margin = mo.min_decision_margin(logits, k)
    print(f"  checker routing done at {time.time() - t0:.1f} s; decision margin {margin:.2e}", flush=True)
    assert margin > 2e-5, "this seed must keep every routing decision clear of fp32 rounding"
    row = mo.dispatch_plan(idx, E, C)
    assert (read_ws(torch, tm, cfg, ws, tm.TM_MOE_WS_TOP_IDX, torch.int32).reshape(-1, k) == idx).all()
    assert (read_ws(torch, tm, cfg, ws, tm.TM_MOE_WS_SLOT_ROW, torch.int32).reshape(-1, k) == library_row(cfg, row)).all()
    assert rel_err(read_ws(torch, tm, cfg, ws, tm.TM_MOE_WS_GATES, torch.float32), gates.reshape(-1)) <= 1e-5
    # the one local expert serves all 16 buffers: rows in checker order
    buf = np.zeros((E * C, h))
    gate_of_row, tok_of_row = np.zeros(E * C), np.full(E * C, -1)
    for t in range(T):
        for i in range(k):
            if row[t, i] >= 0:
                buf[row[t, i]], gate_of_row[row[t, i]], tok_of_row[row[t, i]] = c[t], gates[t, i], t
    u = buf @ w1.T + b1
    g = so.gelu_fwd(u, cfg.act)
    print(f"  checker first expert product done at {time.time() - t0:.1f} s", flush=True)
    rng = np.random.default_rng(9)
    # forward and input gradient on sampled tokens (kept and dropped alike)
    d_o = np.where(tok_of_row[:, None] >= 0, gate_of_row[:, None] * dout[np.maximum(tok_of_row, 0)], 0.0)
    toks = np.concatenate([rng.choice(T, 12, replace=False), np.where((row < 0).any(axis=1))[0][:4]])
    got_out, got_dc = to_host(out), to_host(dc)
    want_out, want_dc = np.zeros((len(toks), h)), np.zeros((len(toks), h))
    for a, t in enumerate(toks):
        dgate = np.zeros(k)
        for i in range(k):
            r = row[t, i]
            if r < 0:
                continue
            o_r = g[r] @ w2.T + b2
            want_out[a] += gates[t, i] * o_r
            dgate[i] = dout[t] @ o_r
            du = so.gelu_bwd(d_o[r] @ w2, u[r], cfg.act)
            want_dc[a] += du @ w1
        dch = gates[t] * (dgate - (gates[t] * dgate).sum())
        want_dc[a] += dch @ wr[idx[t]]
    e_out, e_dc = rel_err(got_out[toks], want_out), rel_err(got_dc[toks], want_dc)
    print(f"  sampled tokens: out {e_out:.3e} dc {e_dc:.3e} at {time.time() - t0:.1f} s", flush=True)
    assert e_out <= TOL_BF16 and e_dc <= TOL_BF16
    # weight gradients on sampled rows
    hs, fs = rng.choice(h, 24, replace=False), rng.choice(f, 24, replace=False)
    off2, off1 = layout["w_fc2.0"][0], layout["w_fc1.0"][0]
    got_w2 = np.stack([to_host(grads[off2 + j * f:off2 + (j + 1) * f]) for j in hs])
    assert rel_err(got_w2, d_o[:, hs].T @ g) <= TOL_BF16
    du_fs = so.gelu_bwd(d_o @ w2[:, fs], u[:, fs], cfg.act)
    got_w1 = np.stack([to_host(grads[off1 + j * h:off1 + (j + 1) * h]) for j in fs])
    assert rel_err(got_w1, du_fs.T @ buf) <= TOL_BF16
    offb = layout["b_fc2.0"][0]
    assert rel_err(to_host(grads[offb:offb + h]), d_o.sum(axis=0)) <= TOL_BF16
    print(f"  weight-gradient samples done at {time.time() - t0:.1f} s", flush=True)
    assert bool(torch.isfinite(grads).all()) and bool(torch.isfinite(out.float()).all())
