"""Pins for the fp64 CPU checker: each test fixes a part of oracle/stage_oracle.py
to something other than itself (finite differences, an independent scalar-loop
evaluation, closed forms, invariants, a library routine, textbook re-assembly of
a tensor-parallel split).  None of these needs a GPU."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import loop_twin
from oracle import stage_oracle as so

RNG = np.random.default_rng(7)

TINY_GPT = si.StageConfig(1, 16, 2, 2, 4, 24, 6, 2, dtype=si.DTYPE_FP32)
TINY_GPT_ERF = TINY_GPT.replace(act=si.ACT_GELU_ERF)
TINY_LLAMA = si.StageConfig(1, 16, 4, 2, 4, 24, 6, 2, dtype=si.DTYPE_FP32, norm=si.NORM_RMSNORM,
                            act=si.ACT_SWIGLU, pos=si.POS_ROTARY, has_bias=0)
TINY_CFGS = [TINY_GPT, TINY_GPT_ERF, TINY_LLAMA]


def _params(cfg, scale=0.3):
    # larger than the training recipe's 0.02 so that every non-linearity is well away from its linear regime
    p = {}
    for name, shape in si.layer_inventory(cfg):
        a = RNG.standard_normal(shape) * scale
        if name.endswith("_gain"):
            a = a + 1.0
        p[name] = a
    return p


# ------------------------------------------------------------------ backward vs finite differences
@pytest.mark.parametrize("cfg", TINY_CFGS)
def test_layer_backward_matches_central_differences(cfg):
    p = _params(cfg)
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    dy = RNG.standard_normal(x.shape)
    y, st = so.layer_fwd(cfg, p, x)
    dx, gr = so.layer_bwd(cfg, p, st, dy)
    assert set(gr) == set(p)

    def loss(pp, xx):
        return float((so.layer_fwd(cfg, pp, xx)[0] * dy).sum())

    eps = 1e-6

    def fd(arr, setter):
        out = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = arr[idx]
            arr[idx] = old + eps
            lp = setter()
            arr[idx] = old - eps
            lm = setter()
            arr[idx] = old
            out[idx] = (lp - lm) / (2 * eps)
        return out

    xv = x.copy()
    num_dx = fd(xv, lambda: loss(p, xv))
    assert np.abs(num_dx - dx).max() <= 1e-6 * max(1.0, np.abs(dx).max())
    for name in p:
        arr = p[name]
        num = fd(arr, lambda: loss(p, x))
        scale = max(1.0, np.abs(gr[name]).max())
        assert np.abs(num - gr[name]).max() <= 1e-6 * scale, name


def test_two_layer_stage_backward_matches_directional_derivative():
    cfg = TINY_LLAMA.replace(n_layers=2)
    layers = [_params(cfg), _params(cfg)]
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    dy = RNG.standard_normal(x.shape)
    y, st = so.stage_fwd(cfg, layers, x)
    dx, grads = so.stage_bwd(cfg, layers, st, dy)
    direction = [{k: RNG.standard_normal(v.shape) for k, v in l.items()} for l in layers]
    dirx = RNG.standard_normal(x.shape)
    analytic = float((dx * dirx).sum()) + sum(float((grads[i][k] * direction[i][k]).sum())
                                              for i in range(2) for k in layers[i])
    eps = 1e-6

    def at(t):
        ls = [{k: v + t * direction[i][k] for k, v in l.items()} for i, l in enumerate(layers)]
        return float((so.stage_fwd(cfg, ls, x + t * dirx)[0] * dy).sum())

    numeric = (at(eps) - at(-eps)) / (2 * eps)
    assert abs(numeric - analytic) <= 1e-6 * max(1.0, abs(analytic))


# ------------------------------------------------------------------ forward vs scalar loops
@pytest.mark.parametrize("cfg", TINY_CFGS)
def test_forward_matches_scalar_loop_evaluation(cfg):
    p = _params(cfg)
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    y, _ = so.layer_fwd(cfg, p, x)
    y_loop = np.array(loop_twin.layer_forward(cfg, {k: v.tolist() for k, v in p.items()}, x.tolist()))
    assert np.abs(y - y_loop).max() <= 1e-12 * max(1.0, np.abs(y).max())


# ------------------------------------------------------------------ softmax / attention
def test_softmax_rows_sum_to_one_and_future_is_exactly_zero():
    q, k = RNG.standard_normal((9, 4)) * 3, RNG.standard_normal((9, 4)) * 3
    p = so.causal_probs(q, k)
    assert np.abs(p.sum(axis=1) - 1.0).max() <= 1e-14
    assert (p[np.triu_indices(9, 1)] == 0.0).all()
    assert p[0, 0] == 1.0


def test_attention_first_row_returns_first_value_exactly():
    q, k, v = (RNG.standard_normal((5, 2, 3, 4)) for _ in range(3))
    ctx = so.attention_fwd(q, k, v)
    assert (ctx[0] == v[0]).all()


def test_attention_zero_queries_give_prefix_means():
    s, b, n, d = 7, 2, 2, 4
    k, v = RNG.standard_normal((s, b, n, d)), RNG.standard_normal((s, b, n, d))
    ctx = so.attention_fwd(np.zeros((s, b, n, d)), k, v)
    prefix = np.cumsum(v, axis=0) / np.arange(1, s + 1)[:, None, None, None]
    assert np.abs(ctx - prefix).max() <= 1e-14


def test_attention_single_position_is_identity_on_v():
    q, k, v = (RNG.standard_normal((1, 3, 2, 4)) for _ in range(3))
    assert (so.attention_fwd(q, k, v) == v).all()


def test_attention_two_positions_closed_form():
    # s = 2: row 1 mixes v0, v1 with a logistic weight of the score gap
    d = 4
    q, k, v = (RNG.standard_normal((2, 1, 1, d)) for _ in range(3))
    ctx = so.attention_fwd(q, k, v)
    gap = (q[1, 0, 0] @ (k[1, 0, 0] - k[0, 0, 0])) / math.sqrt(d)
    w1 = 1.0 / (1.0 + math.exp(-gap))
    assert np.abs(ctx[1, 0, 0] - ((1 - w1) * v[0, 0, 0] + w1 * v[1, 0, 0])).max() <= 1e-14


def test_gqa_equals_mha_with_replicated_kv_heads_and_summed_kv_grads():
    s, b, nq, nkv, d = 6, 2, 4, 2, 4
    q = RNG.standard_normal((s, b, nq, d))
    k, v = RNG.standard_normal((s, b, nkv, d)), RNG.standard_normal((s, b, nkv, d))
    dctx = RNG.standard_normal(q.shape)
    rep = lambda t: np.repeat(t, nq // nkv, axis=2)
    ctx = so.attention_fwd(q, k, v)
    ctx_m = so.attention_fwd(q, rep(k), rep(v))
    assert np.abs(ctx - ctx_m).max() <= 1e-14
    dq, dk, dv = so.attention_bwd(dctx, q, k, v)
    dq_m, dk_m, dv_m = so.attention_bwd(dctx, q, rep(k), rep(v))
    fold = lambda t: t.reshape(s, b, nkv, nq // nkv, d).sum(axis=3)
    assert np.abs(dq - dq_m).max() <= 1e-13
    assert np.abs(dk - fold(dk_m)).max() <= 1e-13
    assert np.abs(dv - fold(dv_m)).max() <= 1e-13


@pytest.mark.parametrize("cfg", [TINY_GPT, TINY_LLAMA])
def test_causality_of_forward_and_backward(cfg):
    p = _params(cfg)
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    i0 = 3
    y, st = so.layer_fwd(cfg, p, x)
    x2 = x.copy()
    x2[i0] += 1.0
    y2, _ = so.layer_fwd(cfg, p, x2)
    assert (y2[:i0] == y[:i0]).all() and np.abs(y2[i0:] - y[i0:]).max() > 1e-3
    dy = RNG.standard_normal(x.shape)
    dx, _ = so.layer_bwd(cfg, p, st, dy)
    dy2 = dy.copy()
    dy2[:i0] += 1.0                   # changing dy at earlier positions must not reach dx at later ones
    dx2, _ = so.layer_bwd(cfg, p, st, dy2)
    assert np.abs(dx2[i0:] - dx[i0:]).max() <= 1e-13


def test_batch_entries_are_independent():
    cfg = TINY_GPT
    p = _params(cfg)
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    y, _ = so.layer_fwd(cfg, p, x)
    x2 = x.copy()
    x2[:, 1] += 1.0
    y2, _ = so.layer_fwd(cfg, p, x2)
    assert (y2[:, 0] == y[:, 0]).all()


# ------------------------------------------------------------------ norms
def test_layernorm_invariants():
    h = 32
    x = RNG.standard_normal((5, h)) * 3 + 2
    gain, off = RNG.standard_normal(h), RNG.standard_normal(h)
    eps = 1e-5
    out, xhat, rstd = so.norm_fwd(x, gain, off, so.NORM_LAYERNORM, eps)
    assert np.abs(xhat.mean(axis=1)).max() <= 1e-14
    var = x.var(axis=1)
    assert np.abs((xhat ** 2).mean(axis=1) - var / (var + eps)).max() <= 1e-13
    out_shift, _, _ = so.norm_fwd(x + 7.0, gain, off, so.NORM_LAYERNORM, eps)
    assert np.abs(out_shift - out).max() <= 1e-12
    # matches the textbook formula evaluated row by row with numpy's own mean/var
    for r in range(5):
        ref = (x[r] - np.mean(x[r])) / np.sqrt(np.var(x[r]) + eps) * gain + off
        assert np.abs(ref - out[r]).max() <= 1e-14
    dout = RNG.standard_normal(x.shape)
    dx, dgain, doff = so.norm_bwd(dout, xhat, rstd, gain, so.NORM_LAYERNORM)
    assert np.abs(dx.sum(axis=1)).max() <= 1e-13
    # sum_h dx*xhat vanishes up to the eps term: rstd * sum(w*xhat) * eps / (var + eps)
    w = dout * gain
    expect = rstd[:, 0] * (w * xhat).sum(axis=1) * eps / (var + eps)
    assert np.abs((dx * xhat).sum(axis=1) - expect).max() <= 1e-13
    dx0 = so.norm_bwd(dout, *so.norm_fwd(x, gain, off, so.NORM_LAYERNORM, 0.0)[1:], gain, so.NORM_LAYERNORM)[0]
    xhat0 = so.norm_fwd(x, gain, off, so.NORM_LAYERNORM, 0.0)[1]
    assert np.abs((dx0 * xhat0).sum(axis=1)).max() <= 1e-12
    assert np.abs(doff - dout.sum(axis=0)).max() <= 1e-14


def test_rmsnorm_invariants():
    h = 32
    x = RNG.standard_normal((5, h)) * 3 + 1
    gain = RNG.standard_normal(h)
    eps = 1e-5
    out, xhat, rstd = so.norm_fwd(x, gain, None, so.NORM_RMSNORM, eps)
    ms = (x ** 2).mean(axis=1)
    assert np.abs((xhat ** 2).mean(axis=1) - ms / (ms + eps)).max() <= 1e-14
    dout = RNG.standard_normal(x.shape)
    dx, _, doff = so.norm_bwd(dout, xhat, rstd, gain, so.NORM_RMSNORM)
    assert doff is None
    # the norm's gradient is orthogonal to x up to the eps term (exactly at eps = 0)
    expect = ((dout * gain) * xhat).sum(axis=1) * eps / (ms + eps)
    assert np.abs((dx * xhat).sum(axis=1) - rstd[:, 0] * expect).max() <= 1e-12
    _, xh0, rs0 = so.norm_fwd(x, gain, None, so.NORM_RMSNORM, 0.0)
    dx0, _, _ = so.norm_bwd(dout, xh0, rs0, gain, so.NORM_RMSNORM)
    assert np.abs((dx0 * x).sum(axis=1)).max() <= 1e-12
    out0, _, _ = so.norm_fwd(x, gain, None, so.NORM_RMSNORM, 0.0)
    out0s, _, _ = so.norm_fwd(5.0 * x, gain, None, so.NORM_RMSNORM, 0.0)
    assert np.abs(out0 - out0s).max() <= 1e-13              # scale invariance at eps = 0


# ------------------------------------------------------------------ activations
def test_gelu_and_silu_special_values():
    z = np.array([0.0])
    for kind in (so.ACT_GELU_TANH, so.ACT_GELU_ERF):
        assert so.gelu_fwd(z, kind)[0] == 0.0
        assert so.gelu_bwd(np.ones(1), z, kind)[0] == 0.5
        big = np.array([12.0])
        assert abs(so.gelu_fwd(big, kind)[0] - 12.0) <= 1e-12
        assert abs(so.gelu_fwd(-big, kind)[0]) <= 1e-12
    u = np.linspace(-6, 6, 2001)
    erf_ref = np.array([0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in u])
    assert np.abs(so.gelu_fwd(u, so.ACT_GELU_ERF) - erf_ref).max() <= 1e-15
    assert np.abs(so.gelu_fwd(u, so.ACT_GELU_TANH) - erf_ref).max() < 1e-3     # the known gap of the tanh form
    assert np.abs(so.gelu_fwd(u, so.ACT_GELU_TANH) - erf_ref).max() > 1e-4
    assert so.swiglu_fwd(z, np.ones(1))[0] == 0.0
    dgate, dup = so.swiglu_bwd(np.ones(1), z, np.ones(1))
    assert dgate[0] == 0.5 and dup[0] == 0.0
    t = np.array([1.7])
    assert abs(so.swiglu_fwd(t, np.array([2.0]))[0] - 2.0 * 1.7 / (1.0 + math.exp(-1.7))) <= 1e-15


# ------------------------------------------------------------------ rotary
def test_rotary_properties():
    s, d = 9, 8
    ang = so.rotary_angles(s, d, 10000.0)
    assert (ang[0] == 0).all() and ang[1, 0] == 1.0
    assert abs(ang[3, 2] - 3 * 10000.0 ** (-4 / 8)) <= 1e-15
    z = RNG.standard_normal((s, 2, 3, d))
    r = so.rotary_apply(z, ang)
    assert (r[0] == z[0]).all()
    pair_norm = lambda t: t[..., : d // 2] ** 2 + t[..., d // 2:] ** 2
    assert np.abs(pair_norm(r) - pair_norm(z)).max() <= 1e-13
    w = RNG.standard_normal(z.shape)
    assert abs((r * w).sum() - (z * so.rotary_apply(w, ang, -1.0)).sum()) <= 1e-12   # backward = transpose
    # explicit 2x2 rotation on one pair
    i, j = 5, 1
    c, sn = math.cos(ang[i, j]), math.sin(ang[i, j])
    assert abs(r[i, 0, 0, j] - (z[i, 0, 0, j] * c - z[i, 0, 0, j + d // 2] * sn)) <= 1e-15
    assert abs(r[i, 0, 0, j + d // 2] - (z[i, 0, 0, j + d // 2] * c + z[i, 0, 0, j] * sn)) <= 1e-15
    # scores depend on relative position only
    q, k = RNG.standard_normal((1, d)), RNG.standard_normal((1, d))
    big = so.rotary_angles(40, d, 10000.0)
    sc = lambda iq, ik: (so.rotary_apply(q, big[iq:iq + 1]) @ so.rotary_apply(k, big[ik:ik + 1]).T).item()
    assert abs(sc(7, 3) - sc(27, 23)) <= 1e-12


# ------------------------------------------------------------------ collectives as identities
def test_tensor_parallel_shards_reassemble_the_unsharded_layer():
    """Column-split Wqkv/W1 (by heads / ffn columns) and row-split Wout/W2 over 2 ranks: the sum of the
    ranks' partial products is the unsharded layer's (what the all-reduce would deliver)."""
    full = si.StageConfig(1, 16, 4, 4, 4, 24, 6, 2, dtype=si.DTYPE_FP32)
    shard = full.replace(n_q_heads=2, n_kv_heads=2, ffn=12)
    p = _params(full)
    x = RNG.standard_normal((full.seq, full.micro_batch, full.hidden))
    y_full, st_full = so.layer_fwd(full, p, x)
    d, A, h = full.head_dim, full.attn_width, full.hidden
    attn_sum = np.zeros_like(x)
    x1_full = st_full["x1"]
    mlp_sum = np.zeros_like(x)
    for r in range(2):
        heads = slice(r * 2 * d, (r + 1) * 2 * d)
        rows = np.r_[np.arange(A)[heads], A + np.arange(A)[heads], 2 * A + np.arange(A)[heads]]
        cols = slice(r * 12, (r + 1) * 12)
        ps = dict(p)
        ps["w_qkv"], ps["b_qkv"] = p["w_qkv"][rows], p["b_qkv"][rows]
        ps["w_out"] = p["w_out"][:, heads]
        ps["w_fc1"], ps["b_fc1"] = p["w_fc1"][cols], p["b_fc1"][cols]
        ps["w_fc2"] = p["w_fc2"][:, cols]
        ps["b_out"] = np.zeros(h)
        ps["b_fc2"] = np.zeros(h)
        _, st = so.layer_fwd(shard, ps, x)
        attn_sum += st["x1"] - x                       # this rank's partial ctx Wout^T
        # MLP partial, evaluated on the full layer's x1 (what every rank holds after the first all-reduce)
        c = st_full["c"]
        g = so.gelu_fwd(c @ ps["w_fc1"].T + ps["b_fc1"], full.act)
        mlp_sum += g @ ps["w_fc2"].T
    assert np.abs(x + attn_sum + p["b_out"] - x1_full).max() <= 1e-13
    assert np.abs(x1_full + mlp_sum + p["b_fc2"] - y_full).max() <= 1e-13


def test_zero_matrices_leave_only_the_residual_path():
    cfg = TINY_GPT
    p = {k: np.zeros(shape) for k, shape in si.layer_inventory(cfg)}
    p["norm1_gain"] += 1.0
    p["norm2_gain"] += 1.0
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    dy = RNG.standard_normal(x.shape)
    y, st = so.layer_fwd(cfg, p, x)
    assert (y == x).all()
    dx, gr = so.layer_bwd(cfg, p, st, dy)
    assert (dx == dy).all()
    col = dy.reshape(-1, cfg.hidden).sum(axis=0)
    assert np.abs(gr["b_fc2"] - col).max() <= 1e-14 and np.abs(gr["b_out"] - col).max() <= 1e-14
    for k in ("w_qkv", "w_out", "w_fc1", "w_fc2", "b_qkv", "b_fc1", "norm1_gain", "norm2_gain"):
        assert (gr[k] == 0).all(), k


# ------------------------------------------------------------------ Adam and bf16 rounding
def test_adam_closed_forms():
    lr, b1, b2, eps = 1e-3, 0.9, 0.999, 1e-8
    p0 = RNG.standard_normal(50)
    g = RNG.standard_normal(50) * 1e-3
    z = np.zeros(50)
    p1, m1, v1 = so.adam_step(p0, g, z, z, 1, lr, b1, b2, eps)
    assert np.abs(p1 - (p0 - lr * g / (np.abs(g) + eps))).max() <= 1e-15
    # constant gradient: the bias-corrected moments stay at g and g^2, so t steps move t times as far
    p, m, v = p0, z, z
    for t in range(1, 6):
        p, m, v = so.adam_step(p, g, m, v, t, lr, b1, b2, eps)
    assert np.abs(p - (p0 - 5 * lr * g / (np.abs(g) + eps))).max() <= 1e-14
    # zero gradient, zero decay: nothing moves
    pz, mz, vz = so.adam_step(p0, z, z, z, 3, lr, b1, b2, eps)
    assert (pz == p0).all() and (mz == 0).all() and (vz == 0).all()
    # decoupled weight decay
    pw, _, _ = so.adam_step(p0, g, z, z, 1, lr, b1, b2, eps, weight_decay=0.1)
    assert np.abs(pw - (p0 * (1 - lr * 0.1) - lr * g / (np.abs(g) + eps))).max() <= 1e-15
    # gradient scale multiplies g before anything else
    ps, ms, vs = so.adam_step(p0, g, z, z, 1, lr, b1, b2, eps, grad_scale=4.0)
    assert np.abs(ms - 0.1 * 4 * g).max() <= 1e-18 and np.abs(vs - 0.001 * 16 * g * g).max() <= 1e-20
    # scalar twin with non-zero state
    m0, v0 = RNG.standard_normal(50) * 1e-4, RNG.random(50) * 1e-6
    pa, ma, va = so.adam_step(p0, g, m0, v0, 7, lr, b1, b2, eps, 0.01, 2.0)
    for i in range(50):
        ref = loop_twin.adam_scalar(p0[i], g[i], m0[i], v0[i], 7, lr, b1, b2, eps, 0.01, 2.0)
        assert abs(pa[i] - ref[0]) <= 1e-15 and abs(ma[i] - ref[1]) <= 1e-18 and abs(va[i] - ref[2]) <= 1e-20


def test_bf16_round_to_nearest_even_on_hand_picked_patterns():
    # (fp32 pattern, expected bf16 pattern)
    cases = [
        (0x3F800000, 0x3F80),   # 1.0 exact
        (0x3F808000, 0x3F80),   # exactly half way, lower neighbour even -> stays
        (0x3F818000, 0x3F82),   # exactly half way, lower neighbour odd -> up to even
        (0x3F808001, 0x3F81),   # just above half way -> up
        (0x3F807FFF, 0x3F80),   # just below half way -> down
        (0xBF818000, 0xBF82),   # sign is carried
        (0x3FFF8000, 0x4000),   # carry into the exponent: 1.9960938 + half ulp -> 2.0
        (0x00000000, 0x0000),
        (0x80000000, 0x8000),
    ]
    pat = np.array([c[0] for c in cases], dtype=np.uint32).view(np.float32)
    got = so.bf16_round_nearest_even(pat)
    assert got.tolist() == [c[1] for c in cases]
    a = (RNG.standard_normal(10000) * 0.02).astype(np.float32)
    back = so.bf16_to_f64(so.bf16_round_nearest_even(a))
    assert (np.abs(back - a) <= 2.0 ** -8 * np.abs(a)).all()   # half an ulp of an 8-bit significand


# ------------------------------------------------------------------ input recipe
def test_input_recipe_is_seeded_and_matches_inventory():
    cfg = si.PRESETS["tiny"]
    a, b = si.make_layer_params(cfg, 1), si.make_layer_params(cfg, 1)
    assert all((a[k] == b[k]).all() for k in a)
    c = si.make_layer_params(cfg, 0)
    assert not (a["w_qkv"] == c["w_qkv"]).all()
    assert si.stage_param_count(cfg) == 1579520
    assert si.stage_param_count(si.PRESETS["gpt175b"]) == 2718922752
    flat = si.make_flat_params(cfg)
    views = si.split_flat(cfg, flat)
    assert (views[1]["w_fc2"] == a["w_fc2"]).all()
    bf = si.make_layer_params(si.PRESETS["tiny"].replace(dtype=si.DTYPE_BF16), 0)
    assert (bf["w_qkv"].view(np.uint32) & 0xFFFF == 0).all()
    assert (si.from_bf16_bits(si.bf16_bits(bf["w_qkv"])) == bf["w_qkv"]).all()
    x = si.make_x(cfg)
    assert x.shape == (128, 2, 256) and abs(float(x.std()) - 1.0) < 0.01


# ----------------------------------------------------------------------------- whole iteration (section 8.1 profiles)
def test_micro_batch_gradients_add_and_equal_one_concatenated_batch():
    """Two micro-batches of one entry each give the same parameter gradients as one micro-batch holding both
    entries (entries are independent and gradients are sums over tokens), and the same outputs per entry."""
    cfg = si.PRESETS["tiny"].replace(n_layers=1, seq=6, hidden=16, n_q_heads=2, n_kv_heads=2, head_dim=8, ffn=24,
                                     micro_batch=1)
    layers = [si.make_layer_params(cfg, 0)]
    xs = [si.make_x(cfg, seed=s) for s in (5, 6)]
    dys = [si.make_dy(cfg, seed=s) for s in (5, 6)]
    ys, dxs, total = so.accumulate_micro_batches(cfg, layers, xs, dys)
    both = cfg.replace(micro_batch=2)
    xb = np.concatenate(xs, axis=1)
    dyb = np.concatenate(dys, axis=1)
    y, st = so.stage_fwd(both, layers, xb)
    dx, grads = so.stage_bwd(both, layers, st, dyb)
    assert np.allclose(np.concatenate(ys, axis=1), y, rtol=0, atol=1e-12)
    assert np.allclose(np.concatenate(dxs, axis=1), dx, rtol=0, atol=1e-12)
    for k in grads[0]:
        assert np.allclose(total[0][k], grads[0][k], rtol=1e-12, atol=1e-15), k


def test_clipping_factor_by_hand():
    assert so.grad_sq_sum(np.array([3.0, -4.0])) == 25.0
    assert so.clip_scale(25.0, 10.0) == 1.0                      # norm 5 under the limit
    assert abs(so.clip_scale(25.0, 1.0) - 1.0 / (5.0 + 1e-6)) < 1e-15
    assert so.clip_scale(25.0, 0.0) == 1.0                       # switched off
    g = np.array([3.0, -4.0]) * so.clip_scale(25.0, 1.0)
    assert abs(np.sqrt(so.grad_sq_sum(g)) - 1.0) < 1e-6          # the clipped gradient has the limit as its norm


def test_optimizer_slices_tile_the_state_once():
    for n, dp in ((100, 3), (96, 3), (7, 8), (1 << 20, 7), (2718922752, 3)):
        covered = 0
        for r in range(dp):
            first, count = so.optimizer_slice(n, dp, r)
            assert first == covered or count == 0
            assert count == 0 or first % 8 == 0
            covered += count
        assert covered == n


def test_iteration_update_touches_only_its_slice_and_folds_both_factors():
    rng = np.random.default_rng(3)
    n = 50
    p, g, m = rng.standard_normal(n), rng.standard_normal(n), rng.standard_normal(n) * 0.1
    v = rng.random(n) * 0.01
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
    p2, m2, v2, factor, first, count = so.iteration_update(p, g, m, v, 4, hp, max_norm=0.5, n_micro=2, dp=3, rank=1)
    assert (first, count) == (24, 24)
    norm_avg = np.sqrt(np.sum((g / 2) ** 2))
    assert abs(factor - 0.5 * 0.5 / (norm_avg + 1e-6)) < 1e-15   # 1/n_micro times c / (norm of the average + eps)
    keep = np.r_[0:24, 48:50]
    assert np.array_equal(p2[keep], p[keep]) and np.array_equal(m2[keep], m[keep]) and np.array_equal(v2[keep], v[keep])
    pe, me, ve = so.adam_step(p[24:48], g[24:48] * factor, m[24:48], v[24:48], 4, **hp)
    assert np.allclose(p2[24:48], pe, rtol=0, atol=1e-15) and np.allclose(m2[24:48], me) and np.allclose(v2[24:48], ve)


# ----------------------------------------------------------------------------- first / last stage layers (section 6.1)
from oracle import roles_oracle as ro  # noqa: E402


def _fd(f, a, eps=1e-6):
    """Central finite-difference gradient of the scalar function f with respect to array a."""
    g = np.zeros_like(a)
    it = np.nditer(a, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = a[i]
        a[i] = old + eps
        fp = f()
        a[i] = old - eps
        fm = f()
        a[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def test_embedding_is_a_row_lookup_and_its_gradient_a_one_hot_product():
    rng = np.random.default_rng(1)
    s, b, h, v_local, v0, n_pos = 5, 3, 4, 6, 10, 8
    w, pos = rng.standard_normal((v_local, h)), rng.standard_normal((n_pos, h))
    tokens = rng.integers(8, 18, size=(s, b))            # ids 8..17: some below, some inside 10..15, some above
    assert ((tokens < v0).any() and (tokens >= v0 + v_local).any() and ((tokens >= v0) & (tokens < v0 + v_local)).any())
    x0 = ro.embedding_fwd(tokens, w, v0, pos)
    for i in range(s):
        for n in range(b):
            row = w[tokens[i, n] - v0] if v0 <= tokens[i, n] < v0 + v_local else 0.0
            assert np.array_equal(x0[i, n], row + pos[i])
    assert np.allclose(ro.embedding_fwd(tokens, w, v0, None), x0 - pos[:s, None, :], rtol=0, atol=1e-15)
    dx0 = rng.standard_normal((s, b, h))
    dw, dp = ro.embedding_bwd(dx0, tokens, v_local, v0, n_pos)
    onehot = (tokens.reshape(-1, 1) - v0 == np.arange(v_local)[None, :]).astype(np.float64)   # [T, V_local]
    assert np.allclose(dw, onehot.T @ dx0.reshape(-1, h), rtol=0, atol=1e-14)
    assert np.allclose(dp[:s], dx0.sum(axis=1)) and not dp[s:].any()
    assert ro.embedding_bwd(dx0, tokens, v_local, v0, 0)[1] is None
    # gradient of a scalar function of x0 by finite differences
    c = rng.standard_normal((s, b, h))
    gw = _fd(lambda: float((ro.embedding_fwd(tokens, w, v0, pos) * c).sum()), w)
    gp = _fd(lambda: float((ro.embedding_fwd(tokens, w, v0, pos) * c).sum()), pos)
    dw2, dp2 = ro.embedding_bwd(c, tokens, v_local, v0, n_pos)
    assert np.allclose(gw, dw2, atol=1e-8) and np.allclose(gp, dp2, atol=1e-8)


def test_cross_entropy_closed_forms():
    T, v_local, v0 = 4, 8, 16
    targets = np.array([16, 23, 3, 40])                   # two inside the shard, one below, one above
    const = np.full((T, v_local), 1.5)
    loss_t, probs = ro.xent_fwd(const, targets, v0)
    assert np.allclose(loss_t, [np.log(8), np.log(8), 1.5 + np.log(8), 1.5 + np.log(8)], rtol=0, atol=1e-14)
    assert np.allclose(probs, 1.0 / 8)
    big = np.zeros((T, v_local))
    big[np.arange(T), [0, 7, 2, 5]] = 10.0                # one dominant logit per row; rows 0, 1 hit their target
    loss_t, probs = ro.xent_fwd(big, targets, v0)
    tail = np.log1p(7 * np.exp(-10.0))
    assert np.allclose(loss_t[:2], tail, rtol=1e-9, atol=0) and np.allclose(loss_t[2:], 10.0 + tail, rtol=0, atol=1e-12)
    assert np.allclose(probs.sum(axis=1), 1.0)
    d = ro.xent_bwd(probs, targets, v0, np.ones(T))
    assert np.allclose(d.sum(axis=1), [0.0, 0.0, 1.0, 1.0], atol=1e-14)   # rows with a local target sum to zero
    shifted, _ = ro.xent_fwd(big + 123.0, targets, v0)    # a shift moves only the rows whose target is elsewhere
    assert np.allclose(shifted[:2], loss_t[:2], atol=1e-9) and np.allclose(shifted[2:], loss_t[2:] + 123.0)


def test_head_gradients_by_finite_differences():
    rng = np.random.default_rng(2)
    s, b, h, v_local, v0 = 3, 2, 6, 5, 7
    for kind in (so.NORM_LAYERNORM, so.NORM_RMSNORM):
        y = rng.standard_normal((s, b, h))
        gain, offset = 1.0 + 0.1 * rng.standard_normal(h), 0.1 * rng.standard_normal(h)
        off = offset if kind == so.NORM_LAYERNORM else None
        w = 0.5 * rng.standard_normal((v_local, h))
        targets = rng.integers(5, 14, size=(s, b))        # ids 5..13 against the shard 7..11
        loss, st = ro.head_fwd(kind, 1e-5, y, gain, off, w, targets, v0)
        dy, dgain, doffset, dw = ro.head_bwd(kind, st, gain, w, targets, v0)
        f = lambda: ro.head_fwd(kind, 1e-5, y, gain, off, w, targets, v0)[0]
        assert np.allclose(_fd(f, y), dy, atol=1e-8)
        assert np.allclose(_fd(f, gain), dgain, atol=1e-8)
        assert np.allclose(_fd(f, w), dw, atol=1e-8)
        if kind == so.NORM_LAYERNORM:
            assert np.allclose(_fd(f, offset), doffset, atol=1e-8)
        else:
            assert doffset is None
        # a loss gradient of 2 doubles everything
        dy2, _, _, dw2 = ro.head_bwd(kind, st, gain, w, targets, v0, dloss=2.0)
        assert np.allclose(dy2, 2 * dy) and np.allclose(dw2, 2 * dw)


def test_vocabulary_shards_reassemble_the_full_embedding_and_the_full_softmax_pieces():
    """Summing the ranks' embedding outputs gives the full-table lookup; the ranks' sum-exp and target-logit
    pieces add up to the full cross-entropy (what the served-locally all-reduces would have combined)."""
    rng = np.random.default_rng(4)
    s, b, h, V, tp = 4, 2, 3, 12, 3
    table = rng.standard_normal((V, h))
    tokens = rng.integers(0, V, size=(s, b))
    full = ro.embedding_fwd(tokens, table, 0, None)
    parts = sum(ro.embedding_fwd(tokens, table[r * 4:(r + 1) * 4], r * 4, None) for r in range(tp))
    assert np.array_equal(full, parts)
    logits = rng.standard_normal((s * b, V))
    targets = rng.integers(0, V, size=s * b)
    full_loss, _ = ro.xent_fwd(logits, targets, 0)
    sumexp, picked = np.zeros(s * b), np.zeros(s * b)
    for r in range(tp):
        lt, _ = ro.xent_fwd(logits[:, r * 4:(r + 1) * 4], targets, r * 4)
        inside = (targets >= r * 4) & (targets < r * 4 + 4)
        lse_r = lt + np.where(inside, logits[np.arange(s * b), targets], 0.0)
        sumexp += np.exp(lse_r)
        picked += np.where(inside, logits[np.arange(s * b), targets], 0.0)
    assert np.allclose(np.log(sumexp) - picked, full_loss, atol=1e-12)


# ------------------------------------------------------------------ record / replay layer of the sandbox (section 4.2)
from oracle import sandbox_oracle as sb  # noqa: E402


@pytest.mark.parametrize("cfg", [TINY_GPT, TINY_LLAMA])
def test_hooked_layer_with_no_peers_is_the_plain_layer(cfg):
    cfg2 = cfg.replace(n_layers=2)
    layers = [_params(cfg2), _params(cfg2)]
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    dy = RNG.standard_normal(x.shape)
    y0, st0 = so.stage_fwd(cfg2, layers, x)
    dx0, g0 = so.stage_bwd(cfg2, layers, st0, dy)
    y1, st1 = sb.stage_fwd(cfg2, layers, x, sb.PassThrough())
    dx1, g1 = sb.stage_bwd(cfg2, layers, st1, dy, sb.PassThrough())
    assert np.abs(y0 - y1).max() <= 1e-13 and np.abs(dx0 - dx1).max() <= 1e-13
    for a, b in zip(g0, g1):
        for k in a:
            assert np.abs(a[k] - b[k]).max() <= 1e-13, k


def _tp_shards(full, p, n_ranks):
    """Megatron split of one layer: heads / ffn columns over the ranks; norm parameters and the biases of the
    row-parallel maps replicated (those biases are added once, after the all-reduce)."""
    d, A = full.head_dim, full.attn_width
    hpr, fpr = full.n_q_heads // n_ranks, full.ffn // n_ranks
    out = []
    for r in range(n_ranks):
        heads = np.arange(r * hpr * d, (r + 1) * hpr * d)
        rows = np.r_[heads, A + heads, 2 * A + heads]
        cols = slice(r * fpr, (r + 1) * fpr)
        ps = dict(p)
        ps["w_qkv"], ps["b_qkv"] = p["w_qkv"][rows], p["b_qkv"][rows]
        ps["w_out"] = p["w_out"][:, heads]
        ps["w_fc1"], ps["b_fc1"] = p["w_fc1"][cols], p["b_fc1"][cols]
        ps["w_fc2"] = p["w_fc2"][:, cols]
        out.append(ps)
    return out


def test_replay_reproduces_a_rank_of_a_real_tensor_parallel_group():
    """Two ranks run the hooked stage as a REAL group (their partial sums are added), rank 0 records every
    scope.  The group's result is the unsharded layer's; rank 0 replaying ALONE gets its own outputs and
    gradients of the group run bit for bit; with only the pipeline scope on the boundary and the tensor
    scope left to its (absent) peers, it does not."""
    import threading
    full = si.StageConfig(2, 16, 4, 4, 4, 24, 6, 2, dtype=si.DTYPE_FP32)
    shard = full.replace(n_q_heads=2, n_kv_heads=2, ffn=12)
    layers_full = [_params(full), _params(full)]
    per_rank = list(zip(*[_tp_shards(full, p, 2) for p in layers_full]))   # [rank][layer]
    x = RNG.standard_normal((full.seq, full.micro_batch, full.hidden))
    dy = RNG.standard_normal(x.shape)
    group = sb.ThreadGroup(2)
    rec = sb.Recorder(group.member(0), sb.SCOPE_TP | sb.SCOPE_PP)
    comms = [rec, group.member(1)]
    res = [None, None]

    def run(r):
        y, st = sb.stage_fwd(shard, per_rank[r], x, comms[r])
        dx, gr = sb.stage_bwd(shard, per_rank[r], st, dy, comms[r])
        res[r] = (y, dx, gr)

    th = [threading.Thread(target=run, args=(r,)) for r in range(2)]
    [t.start() for t in th]
    [t.join(60) for t in th]
    assert res[0] is not None and res[1] is not None
    # the real group computes the unsharded stage
    y_full, st_full = so.stage_fwd(full, layers_full, x)
    dx_full, g_full = so.stage_bwd(full, layers_full, st_full, dy)
    for r in range(2):
        assert np.abs(res[r][0] - y_full).max() <= 1e-12 and np.abs(res[r][1] - dx_full).max() <= 1e-12
    heads0 = np.arange(0, 2 * full.head_dim)
    assert np.abs(res[0][2][1]["w_out"] - g_full[1]["w_out"][:, heads0]).max() <= 1e-12
    assert np.abs(res[0][2][0]["w_fc1"] - g_full[0]["w_fc1"][:12]).max() <= 1e-12
    # tape: recv x, 2 all-reduces per layer forward, recv dy, 2 per layer backward
    kinds = [(e[0], e[2]) for e in rec.tape]
    assert kinds == [(sb.RECV, sb.SITE_X)] + [(sb.ALL_REDUCE, sb.SITE_ATTN_OUT), (sb.ALL_REDUCE, sb.SITE_MLP_OUT)] * 2 + \
        [(sb.RECV, sb.SITE_DY)] + [(sb.ALL_REDUCE, sb.SITE_D_MLP_IN), (sb.ALL_REDUCE, sb.SITE_D_ATTN_IN)] * 2
    # rank 0 alone, every recorded scope on the boundary; the arguments are NOT the real x / dy: the tape supplies them
    rp = sb.Replayer(rec.tape, sb.SCOPE_TP | sb.SCOPE_PP)
    junk = np.zeros_like(x)
    y, st = sb.stage_fwd(shard, per_rank[0], junk, rp)
    dx, gr = sb.stage_bwd(shard, per_rank[0], st, junk, rp)
    assert (y == res[0][0]).all() and (dx == res[0][1]).all()
    for l in range(2):
        for k in gr[l]:
            assert (gr[l][k] == res[0][2][l][k]).all(), k
    assert rp.at == len(rec.tape) and rp.skipped == 2          # both sends skipped
    # boundary = pipeline scope only: the tensor-parallel sums lack rank 1's share
    rp2 = sb.Replayer(rec.tape, sb.SCOPE_PP)
    y2, _ = sb.stage_fwd(shard, per_rank[0], junk, rp2)
    assert np.abs(y2 - y_full).max() > 1e-3 and rp2.at == 1


def test_replay_refuses_a_different_call_sequence_and_skips_barriers():
    cfg = TINY_GPT
    layers = [_params(cfg)]
    x = RNG.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))
    rec = sb.Recorder(sb.PassThrough(), sb.SCOPE_PP | sb.SCOPE_DP)
    y, st = sb.stage_fwd(cfg, layers, x, rec)
    g = RNG.standard_normal(50)
    out = sb.grad_sync(g, rec)
    assert (out == g).all() and len(rec.tape) == 2                    # recv x and the gradient all-reduce; no barrier, no send
    rp = sb.Replayer(rec.tape, sb.SCOPE_PP | sb.SCOPE_DP)
    with pytest.raises(sb.ReplayMismatch):
        sb.stage_bwd(cfg, layers, st, x, rp)                           # asks for dy where the tape holds x
    rp = sb.Replayer(rec.tape, sb.SCOPE_DP)
    assert (sb.grad_sync(np.zeros(50), rp) == g).all() and rp.skipped == 1
    with pytest.raises(sb.ReplayMismatch):
        sb.grad_sync(np.zeros(50), rp)                                 # tape exhausted
    rp = sb.Replayer(rec.tape, sb.SCOPE_DP)
    with pytest.raises(sb.ReplayMismatch):
        sb.grad_sync(np.zeros(51), rp)                                 # other shape


# ------------------------------------------------------------------ mixture-of-experts MLP shard
from oracle import moe_oracle as mo  # noqa: E402


def _moe_params(h, f, E, ep, bias=True, scale=0.3):
    p = {"w_router": RNG.standard_normal((E, h)) * scale}
    for j in range(E // ep):
        p[f"w_fc1.{j}"] = RNG.standard_normal((f, h)) * scale
        p[f"w_fc2.{j}"] = RNG.standard_normal((h, f)) * scale
        if bias:
            p[f"b_fc1.{j}"] = RNG.standard_normal(f) * scale
            p[f"b_fc2.{j}"] = RNG.standard_normal(h) * scale
    return p


@pytest.mark.parametrize("E,ep,k,cap,bias", [(4, 1, 2, 5, True), (6, 3, 2, 3, False), (4, 2, 1, 4, True), (3, 1, 3, 9, True)])
def test_moe_backward_matches_central_differences(E, ep, k, cap, bias):
    T, h, f = 9, 6, 8
    p = _moe_params(h, f, E, ep, bias)
    c = RNG.standard_normal((T, h))
    dout = RNG.standard_normal((T, h))
    out, st = mo.moe_fwd(c, p, E, ep, k, cap, so.ACT_GELU_TANH)
    assert mo.min_decision_margin(st["logits"], min(k, E - 1)) > 2e-5      # the routing is constant around this point
    dc, gr = mo.moe_bwd(dout, p, st, E, ep, k, cap, so.ACT_GELU_TANH)
    loss = lambda cc, pp: float((mo.moe_fwd(cc, pp, E, ep, k, cap, so.ACT_GELU_TANH)[0] * dout).sum())
    eps = 1e-6
    for _ in range(12):
        t, j = RNG.integers(T), RNG.integers(h)
        cp, cm = c.copy(), c.copy()
        cp[t, j] += eps
        cm[t, j] -= eps
        fd = (loss(cp, p) - loss(cm, p)) / (2 * eps)
        assert abs(fd - dc[t, j]) <= 1e-6 * max(1.0, abs(fd)), ("dc", t, j)
    for name in p:
        for _ in range(6):
            pos = tuple(RNG.integers(n) for n in p[name].shape)
            pp, pm = {k_: v.copy() for k_, v in p.items()}, {k_: v.copy() for k_, v in p.items()}
            pp[name][pos] += eps
            pm[name][pos] -= eps
            fd = (loss(c, pp) - loss(c, pm)) / (2 * eps)
            assert abs(fd - gr[name][pos]) <= 1e-6 * max(1.0, abs(fd)), (name, pos)


def test_moe_with_one_expert_is_the_dense_mlp():
    T, h, f = 7, 6, 10
    p = _moe_params(h, f, 1, 1)
    c = RNG.standard_normal((T, h))
    out, st = mo.moe_fwd(c, p, 1, 1, 1, T, so.ACT_GELU_ERF)
    dense = so.gelu_fwd(c @ p["w_fc1.0"].T + p["b_fc1.0"], so.ACT_GELU_ERF) @ p["w_fc2.0"].T + p["b_fc2.0"]
    assert np.abs(out - dense).max() <= 1e-13 and (st["gates"] == 1.0).all()
    dout = RNG.standard_normal((T, h))
    dc, gr = mo.moe_bwd(dout, p, st, 1, 1, 1, T, so.ACT_GELU_ERF)
    du = so.gelu_bwd(dout @ p["w_fc2.0"], c @ p["w_fc1.0"].T + p["b_fc1.0"], so.ACT_GELU_ERF)
    assert np.abs(dc - du @ p["w_fc1.0"]).max() <= 1e-13
    assert np.abs(gr["w_fc1.0"] - du.T @ c).max() <= 1e-13 and np.abs(gr["w_router"]).max() == 0.0


def test_moe_choosing_every_expert_is_the_softmax_mixture():
    T, h, f, E = 6, 5, 7, 4
    p = _moe_params(h, f, E, 1)
    c = RNG.standard_normal((T, h))
    out, st = mo.moe_fwd(c, p, E, 1, E, T, so.ACT_GELU_TANH)
    lg = c @ p["w_router"].T
    sm = np.exp(lg) / np.exp(lg).sum(axis=1, keepdims=True)
    want = np.zeros((T, h))
    for e in range(E):
        want += sm[:, e:e + 1] * (so.gelu_fwd(c @ p[f"w_fc1.{e}"].T + p[f"b_fc1.{e}"], so.ACT_GELU_TANH) @ p[f"w_fc2.{e}"].T
                                  + p[f"b_fc2.{e}"])
    assert np.abs(out - want).max() <= 1e-12
    assert np.abs(st["gates"].sum(axis=1) - 1.0).max() <= 1e-15
    assert (np.diff(np.take_along_axis(lg, st["idx"], axis=1), axis=1) <= 0).all()      # decreasing logit


def test_moe_full_buffer_drops_later_tokens_and_ties_go_to_the_lower_index():
    T, h, f, E, C = 6, 4, 5, 3, 2
    p = _moe_params(h, f, E, 1)
    p["w_router"] = np.zeros((E, h))
    p["w_router"][1, 0] = 5.0                       # expert 1 wins wherever c[:, 0] > 0; experts 0 and 2 tie at 0
    c = np.abs(RNG.standard_normal((T, h))) + 0.1
    out, st = mo.moe_fwd(c, p, E, 1, 2, C, so.ACT_GELU_TANH)
    assert (st["idx"] == np.array([1, 0])).all()    # the tie between experts 0 and 2 goes to 0
    assert (st["row"][:C, 0] == C * 1 + np.arange(C)).all() and (st["row"][C:] == -1).all()
    assert (out[C:] == 0).all() and np.abs(out[:C]).min() > 0
    assert (st["buf"][2 * C:] == 0).all()           # expert 2's buffer stays empty
    dout = RNG.standard_normal((T, h))
    dc, gr = mo.moe_bwd(dout, p, st, E, 1, 2, C, so.ACT_GELU_TANH)
    assert (dc[C:] == 0).all() and (gr["w_fc1.2"] == 0).all()
    assert np.abs(gr["b_fc2.1"] - (st["gates"][:C, :1] * dout[:C]).sum(axis=0)).max() <= 1e-14


def test_moe_expert_parallel_groups_share_the_local_weights():
    T, h, f, E, ep, k, C = 10, 6, 8, 6, 3, 2, 3
    p = _moe_params(h, f, E, ep)
    c, dout = RNG.standard_normal((T, h)), RNG.standard_normal((T, h))
    out, st = mo.moe_fwd(c, p, E, ep, k, C, so.ACT_GELU_TANH)
    dc, gr = mo.moe_bwd(dout, p, st, E, ep, k, C, so.ACT_GELU_TANH)
    wide = {"w_router": p["w_router"]}
    for e in range(E):
        for name in ("w_fc1", "b_fc1", "w_fc2", "b_fc2"):
            wide[f"{name}.{e}"] = p[f"{name}.{e % (E // ep)}"]
    out2, st2 = mo.moe_fwd(c, wide, E, 1, k, C, so.ACT_GELU_TANH)
    dc2, gr2 = mo.moe_bwd(dout, wide, st2, E, 1, k, C, so.ACT_GELU_TANH)
    assert np.abs(out - out2).max() <= 1e-13 and np.abs(dc - dc2).max() <= 1e-13
    for j in range(E // ep):
        for name in ("w_fc1", "b_fc1", "w_fc2", "b_fc2"):
            total = sum(gr2[f"{name}.{e}"] for e in range(E) if e % (E // ep) == j)
            assert np.abs(gr[f"{name}.{j}"] - total).max() <= 1e-12
