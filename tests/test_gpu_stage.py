"""End-to-end parity of tm_stage_fwd / tm_stage_bwd / tm_adam_step against the fp64 CPU checker,
plus the properties the sandboxed warm-up relies on (overwritable state, reproducible results)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import stage_oracle as so
from tests.gpu_util import TOL_ADAM, TOL_BF16, TOL_FP32, pass_rate, rel_err, require_gpu, stream_ptr, to_dev, to_host
from tests.stage_runner import GpuStage, flatten_grads, oracle_iteration

pytestmark = pytest.mark.gpu

SMALL_GPT = si.StageConfig(2, 256, 2, 2, 128, 512, 200, 2)                     # bf16, ragged sequence, batch 2
SMALL_LLAMA = si.StageConfig(2, 256, 4, 1, 64, 328, 130, 1, norm=si.NORM_RMSNORM, act=si.ACT_SWIGLU,
                             pos=si.POS_ROTARY, has_bias=0)
SMALL_ERF = si.StageConfig(1, 128, 2, 2, 32, 256, 40, 1, act=si.ACT_GELU_ERF)   # plain-ALU attention in bf16
TINY = si.PRESETS["tiny"]
TINY_LLAMA_FP32 = si.StageConfig(1, 64, 4, 2, 16, 96, 33, 2, dtype=si.DTYPE_FP32, norm=si.NORM_RMSNORM,
                                 act=si.ACT_SWIGLU, pos=si.POS_ROTARY, has_bias=0)


@pytest.fixture(scope="module")
def env():
    torch = require_gpu()
    import paper_2412_12636_amd as tm
    return torch, tm


def run_and_compare(torch, tm, cfg, progress=False, tol=None, report=None, adam=True):
    """One iteration on the GPU and on the checker from the same seeded inputs.  tol: the max-norm tolerance of every
    tensor (default: the stated 2e-2 / 1e-4), or a function of the tensor's name.  report: a dict that receives, per
    tensor, (rel_err, pass_rate at the stated tolerance).  adam=False leaves out the optimizer part (whole-state fp64
    copies: too much host memory at the largest shard)."""
    stated = TOL_BF16 if cfg.dtype == si.DTYPE_BF16 else TOL_FP32
    tol_of = tol if callable(tol) else (lambda name, t=(stated if tol is None else tol): t)
    say = progress if callable(progress) else (lambda m: print(m, flush=True))
    flat = si.make_flat_params(cfg)
    x, dy = si.make_x(cfg), si.make_dy(cfg)
    st = GpuStage(torch, tm, cfg, flat)
    y = to_host(st.fwd(to_dev(torch, x, cfg.dtype)))
    dx = to_host(st.bwd(to_dev(torch, dy, cfg.dtype)))
    torch.cuda.synchronize()
    gpu_grads = st.grads.cpu().numpy().astype(np.float64)
    layers = si.split_flat(cfg, flat)
    ry, rdx, rgrads = oracle_iteration(cfg, layers, x, dy, progress)
    errs = {"y": rel_err(y, ry), "dx": rel_err(dx, rdx)}
    rates = {"y": pass_rate(y, ry, stated), "dx": pass_rate(dx, rdx, stated)}
    off = 0
    for l in range(cfg.n_layers):
        for name, shape in si.layer_inventory(cfg):
            n = int(np.prod(shape))
            errs[f"layer{l}.{name}"] = rel_err(gpu_grads[off:off + n], rgrads[l][name].reshape(-1))
            rates[f"layer{l}.{name}"] = pass_rate(gpu_grads[off:off + n], rgrads[l][name].reshape(-1), stated)
            off += n
    worst = max(errs, key=errs.get)
    lowest = min(rates, key=rates.get)
    say(f"worst {worst}: {errs[worst]:.3e}  y {errs['y']:.3e}  dx {errs['dx']:.3e}; elementwise pass rate at "
        f"{stated:g}: lowest {lowest} {rates[lowest]:.5f}, y {rates['y']:.5f}, dx {rates['dx']:.5f}")
    if report is not None:
        report.update({k: (errs[k], rates[k]) for k in errs})
    for k, e in errs.items():
        assert e <= tol_of(k), (k, e, tol_of(k))

    if not adam:
        st.close()
        return errs
    # Adam: fed the GPU's own fp32 gradients on both sides, the master weights must agree to 1e-5
    p0 = flat.astype(np.float64)
    z = np.zeros_like(p0)
    st.adam(step=1)
    torch.cuda.synchronize()
    rp, rm, rv = so.adam_step(p0, gpu_grads, z, z, 1, **{k: si.ADAM_DEFAULTS[k] for k in
                                                         ("lr", "beta1", "beta2", "eps", "weight_decay", "grad_scale")})
    assert rel_err(to_host(st.master_weights()), rp) <= TOL_ADAM
    assert rel_err(to_host(st.m), rm) <= TOL_ADAM and rel_err(to_host(st.v), rv) <= TOL_ADAM
    if cfg.dtype == si.DTYPE_BF16:
        want = so.bf16_round_nearest_even(st.master.cpu().numpy())
        got = st.params.view(torch.int16).cpu().numpy().view(np.uint16)
        assert (got == want).all()
    # chained end to end (checker gradients -> checker Adam): at step 1 the update is lr*g/(|g|+eps),
    # insensitive to small gradient errors except where g is near zero
    cp, _, _ = so.adam_step(p0, flatten_grads(cfg, rgrads), z, z, 1, 1e-3, 0.9, 0.999, 1e-8)
    chained = np.abs(to_host(st.master_weights()) - cp)
    say(f"chained Adam: max |dp| {chained.max():.3e} (lr = 1e-3), mean {chained.mean():.3e}")
    assert chained.max() <= 2.0e-3 + 1e-6      # never more than the two updates pointing opposite ways
    st.close()
    return errs


@pytest.mark.parametrize("cfg", [TINY, TINY_LLAMA_FP32, SMALL_GPT, SMALL_LLAMA, SMALL_ERF],
                         ids=["tiny", "tiny_llama_fp32", "small_gpt", "small_llama", "small_erf"])
def test_stage_iteration_matches_checker(env, cfg):
    torch, tm = env
    print(f"stage parity {cfg}", flush=True)
    run_and_compare(torch, tm, cfg)


def test_gpt6p7b_shard_full_depth(env):
    torch, tm = env
    print("stage parity gpt6p7b (4 layers, full size)", flush=True)
    run_and_compare(torch, tm, si.PRESETS["gpt6p7b"], progress=True)


def test_backward_needs_forward_and_gradients_accumulate(env):
    torch, tm = env
    cfg = SMALL_GPT
    flat = si.make_flat_params(cfg)
    st = GpuStage(torch, tm, cfg, flat)
    x, dy = to_dev(torch, si.make_x(cfg), cfg.dtype), to_dev(torch, si.make_dy(cfg), cfg.dtype)
    with pytest.raises(tm.TmError) as e:
        st.bwd(dy)
    assert e.value.code == tm.TM_ESTATE
    st.fwd(x)
    st.bwd(dy)
    g1 = st.grads.clone()
    st.bwd(dy)
    torch.cuda.synchronize()
    assert rel_err(to_host(st.grads), 2.0 * to_host(g1)) <= 1e-6
    # zero_grads clears the buffer inside the Adam kernel
    st.adam(step=1, zero_grads=1)
    torch.cuda.synchronize()
    assert float(st.grads.abs().max()) == 0.0
    st.close()


def test_overwrite_mode_equals_accumulation_into_zeros(env):
    torch, tm = env
    cfg = SMALL_GPT
    flat = si.make_flat_params(cfg)
    x, dy = to_dev(torch, si.make_x(cfg), cfg.dtype), to_dev(torch, si.make_dy(cfg), cfg.dtype)
    a = GpuStage(torch, tm, cfg, flat)
    a.fwd(x)
    a.bwd(dy)
    b = GpuStage(torch, tm, cfg, flat)
    b.grads.fill_(float("nan"))                 # dead contents: must never be read
    tm.tm_stage_grad_mode(b.handle, True)
    b.fwd(x)
    b.bwd(dy)
    torch.cuda.synchronize()
    assert torch.equal(a.grads, b.grads) and torch.equal(a.dx, b.dx)
    tm.tm_stage_grad_mode(b.handle, False)      # back to accumulation: a second pass doubles the gradients
    b.bwd(dy)
    torch.cuda.synchronize()
    assert rel_err(to_host(b.grads), 2.0 * to_host(a.grads)) <= 1e-6
    a.close()
    b.close()


def test_tuning_changes_speed_only(env):
    """Timing the tile configurations keeps every result bit for bit (each configuration accumulates an
    output element in the same order), overwrites the workspace, and asks for a new forward pass."""
    torch, tm = env
    cfg = SMALL_GPT.replace(hidden=512, ffn=1024, n_q_heads=4, n_kv_heads=4, seq=192)   # every K a multiple of 64
    flat = si.make_flat_params(cfg)
    x, dy = to_dev(torch, si.make_x(cfg), cfg.dtype), to_dev(torch, si.make_dy(cfg), cfg.dtype)
    st = GpuStage(torch, tm, cfg, flat)
    st.fwd(x)
    st.bwd(dy)
    torch.cuda.synchronize()
    y0, dx0, g0 = st.y.clone(), st.dx.clone(), st.grads.clone()
    tm.tm_stage_tune(st.handle, stream_ptr(torch))
    with pytest.raises(tm.TmError) as ei:
        st.bwd(dy)                               # the stash is gone
    assert ei.value.code == tm.TM_ESTATE
    st.grads.zero_()
    st.fwd(x)
    st.bwd(dy)
    torch.cuda.synchronize()
    assert torch.equal(st.y, y0) and torch.equal(st.dx, dx0) and torch.equal(st.grads, g0)
    st.close()


# FC matrices of 4104 x 6152 and 6152 x 4104: 17 x 33 and 25 x 22 tiles of 256 x 192 with ragged last tiles, enough of
# them for the update products' large staggered form; 64 tokens are a single reduction step, 192 are three
WIDE_RAGGED = si.StageConfig(1, 6152, 2, 2, 128, 4104, 64, 1)


@pytest.mark.parametrize("cfg", [SMALL_GPT.replace(n_layers=3), SMALL_GPT.replace(n_layers=3, seq=192),
                                 SMALL_LLAMA.replace(n_layers=2, seq=256), TINY, WIDE_RAGGED, WIDE_RAGGED.replace(seq=192)],
                         ids=["ragged_tokens_flat_sweep", "fused_into_the_products", "fused_llama", "fp32_flat_sweep",
                              "fused_large_staggered_ragged_one_step", "fused_large_staggered_ragged_three_steps"])
def test_backward_with_overlapped_optimizer_equals_the_two_calls(env, cfg):
    """tm_stage_bwd_adam = tm_stage_bwd then tm_adam_step, bit for bit: gradients, master weights, both moments, the
    bf16 copy, the input gradient; two iterations, so that the second forward pass sees updated weights.  With a
    token count that is a multiple of 64 the matrices' updates ride in the weight-gradient products' epilogues and
    the flat sweep covers the vectors between them; otherwise (and for fp32 stages) the flat sweep does it all."""
    torch, tm = env
    flat = si.make_flat_params(cfg)
    x, dy = to_dev(torch, si.make_x(cfg), cfg.dtype), to_dev(torch, si.make_dy(cfg), cfg.dtype)
    a, b = GpuStage(torch, tm, cfg, flat), GpuStage(torch, tm, cfg, flat)
    hp = tm.make_hparams(**si.ADAM_DEFAULTS)
    for st in (a, b):
        tm.tm_stage_grad_mode(st.handle, True)
    for step in (1, 2):
        a.fwd(x)
        a.bwd(dy)
        a.adam(step=step)
        b.fwd(x)
        tm.tm_stage_bwd_adam(b.handle, dy, b.dx, hp, step, stream_ptr(torch))
        torch.cuda.synchronize()
        for name in ("y", "dx", "grads", "master", "m", "v", "params"):
            if getattr(a, name) is not None:                  # fp32 stages have no separate master copy
                assert torch.equal(getattr(a, name), getattr(b, name)), (step, name)
    # transient gradients: the same update, the vectors' gradients stored as before, the matrices' unspecified
    c = GpuStage(torch, tm, cfg, flat)
    tm.tm_stage_grad_mode(c.handle, tm.TM_GRAD_TRANSIENT)
    c.grads.fill_(3.0)
    for step in (1, 2):
        c.fwd(x)
        tm.tm_stage_bwd_adam(c.handle, dy, c.dx, hp, step, stream_ptr(torch))
    torch.cuda.synchronize()
    for name in ("y", "dx", "master", "m", "v", "params"):
        if getattr(a, name) is not None:
            assert torch.equal(getattr(a, name), getattr(c, name)), name
    for name, off, shape in tm.tm_stage_param_layout(cfg):
        if shape[1] == 1:
            assert torch.equal(a.grads[off:off + shape[0]], c.grads[off:off + shape[0]]), name
    with pytest.raises(tm.TmError):
        tm.tm_stage_grad_mode(c.handle, 3)
    a.close()
    b.close()
    c.close()


def test_backward_with_update_rejects_bad_scalars_before_any_launch(env):
    """step < 1 or a beta outside [0, 1) is refused before the first kernel: no state is touched."""
    torch, tm = env
    cfg = SMALL_GPT.replace(seq=192)                     # token count a multiple of 64: the fused update path
    flat = si.make_flat_params(cfg)
    x, dy = to_dev(torch, si.make_x(cfg), cfg.dtype), to_dev(torch, si.make_dy(cfg), cfg.dtype)
    st = GpuStage(torch, tm, cfg, flat)
    tm.tm_stage_grad_mode(st.handle, tm.TM_GRAD_TRANSIENT)
    st.fwd(x)
    torch.cuda.synchronize()
    before = {k: getattr(st, k).clone() for k in ("master", "m", "v", "params", "grads")}
    for hp, step in ((tm.make_hparams(**si.ADAM_DEFAULTS), 0),
                     (tm.make_hparams(**{**si.ADAM_DEFAULTS, "beta2": 1.0}), 1),
                     (tm.make_hparams(**{**si.ADAM_DEFAULTS, "beta1": -0.1}), 1)):
        with pytest.raises(tm.TmError) as e:
            tm.tm_stage_bwd_adam(st.handle, dy, st.dx, hp, step, stream_ptr(torch))
        assert e.value.code == tm.TM_EINVAL
    torch.cuda.synchronize()
    for k, old in before.items():
        assert torch.equal(getattr(st, k), old), k
    # the handle is still good
    tm.tm_stage_bwd_adam(st.handle, dy, st.dx, tm.make_hparams(**si.ADAM_DEFAULTS), 1, stream_ptr(torch))
    torch.cuda.synchronize()
    assert not torch.equal(st.master, before["master"])
    st.close()


def test_backward_on_one_stream_equals_backward_on_two(env, monkeypatch):
    """Everything on the caller's stream (default) against the weight-gradient products forked onto the internal
    second stream (TM_BWD_STREAMS=2): same bits."""
    torch, tm = env
    cfg = SMALL_GPT.replace(n_layers=3)
    flat = si.make_flat_params(cfg)
    x, dy = to_dev(torch, si.make_x(cfg), cfg.dtype), to_dev(torch, si.make_dy(cfg), cfg.dtype)
    a, b = GpuStage(torch, tm, cfg, flat), GpuStage(torch, tm, cfg, flat)
    a.fwd(x)
    a.bwd(dy)
    torch.cuda.synchronize()
    monkeypatch.setenv("TM_BWD_STREAMS", "2")
    b.fwd(x)
    b.bwd(dy)
    torch.cuda.synchronize()
    monkeypatch.delenv("TM_BWD_STREAMS")
    assert torch.equal(a.grads, b.grads) and torch.equal(a.dx, b.dx)
    a.close()
    b.close()


@pytest.mark.parametrize("cfg", [SMALL_GPT, SMALL_LLAMA], ids=["small_gpt", "small_llama"])
def test_whole_iteration_of_several_micro_batches(env, cfg):
    """Three micro-batches (first stored, the others accumulated), the squared gradient norm, the clipping
    factor and the Adam update of one data-parallel rank's slice, against the checker's whole iteration
    (section 8.1 profiles: several micro-batches per iteration, distributed optimizer)."""
    torch, tm = env
    n_micro, dp, rank, max_norm = 3, 3, 1, 0.05
    flat = si.make_flat_params(cfg)
    layers = si.split_flat(cfg, flat)
    xs = [si.make_x(cfg, seed=100 + i) for i in range(n_micro)]
    dys = [si.make_dy(cfg, seed=100 + i) for i in range(n_micro)]
    st = GpuStage(torch, tm, cfg, flat)
    st.grads.fill_(float("nan"))                         # the first micro-batch must not read it
    for i in range(n_micro):
        tm.tm_stage_grad_mode(st.handle, i == 0)
        st.fwd(to_dev(torch, xs[i], cfg.dtype))
        st.bwd(to_dev(torch, dys[i], cfg.dtype))
    sq = torch.zeros(1, dtype=torch.float64, device="cuda")
    tm.tm_stage_grad_sq_sum(st.handle, sq, stream_ptr(torch))
    torch.cuda.synchronize()
    gpu_grads = st.grads.cpu().numpy().astype(np.float64)
    _, _, rgrads = so.accumulate_micro_batches(cfg, layers, xs, dys)
    ref_grads = flatten_grads(cfg, rgrads)
    off = 0
    for l in range(cfg.n_layers):
        for name, shape in si.layer_inventory(cfg):
            n = int(np.prod(shape))
            assert rel_err(gpu_grads[off:off + n], ref_grads[off:off + n]) <= TOL_BF16, (l, name)
            off += n
    # the squared norm: tight against the GPU's own gradients, bf16-loose against the checker's
    assert abs(float(sq.item()) - so.grad_sq_sum(gpu_grads)) <= 1e-6 * so.grad_sq_sum(gpu_grads)
    assert abs(float(sq.item()) - so.grad_sq_sum(ref_grads)) <= 2 * TOL_BF16 * so.grad_sq_sum(ref_grads)
    # the host forms the factor as the checker does; it clips in this set-up
    factor = (1.0 / n_micro) * so.clip_scale(float(sq.item()) / n_micro ** 2, max_norm)
    assert factor < 1.0 / n_micro
    first, count = so.optimizer_slice(st.n, dp, rank)
    hp_kw = {**si.ADAM_DEFAULTS, "grad_scale": factor}
    before = {k: getattr(st, k).clone() for k in ("master", "m", "v", "params")}
    tm.tm_adam_step_range(st.handle, first, count, tm.make_hparams(**hp_kw), 1, stream_ptr(torch))
    torch.cuda.synchronize()
    hp = {k: si.ADAM_DEFAULTS[k] for k in ("lr", "beta1", "beta2", "eps", "weight_decay")}
    z = np.zeros(st.n)
    rp, rm, rv, rfactor, rfirst, rcount = so.iteration_update(flat.astype(np.float64), gpu_grads, z, z, 1, hp, max_norm,
                                                              n_micro, dp, rank)
    assert (rfirst, rcount) == (first, count) and abs(rfactor - factor) <= 1e-9 * factor
    assert rel_err(to_host(st.master), rp) <= TOL_ADAM
    assert rel_err(to_host(st.m), rm) <= TOL_ADAM and rel_err(to_host(st.v), rv) <= TOL_ADAM
    outside = torch.ones(st.n, dtype=torch.bool, device="cuda")
    outside[first:first + count] = False
    for k, old in before.items():                        # nothing outside the slice moved
        assert torch.equal(getattr(st, k)[outside], old[outside]), k
    assert not torch.equal(st.master[first:first + count], before["master"][first:first + count])
    with pytest.raises(tm.TmError) as e:
        tm.tm_adam_step_range(st.handle, 4, 8, tm.make_hparams(**hp_kw), 1, stream_ptr(torch))
    assert e.value.code == tm.TM_EALIGN
    with pytest.raises(tm.TmError) as e:
        tm.tm_adam_step_range(st.handle, 0, st.n + 8, tm.make_hparams(**hp_kw), 1, stream_ptr(torch))
    assert e.value.code == tm.TM_EINVAL
    st.close()


def test_two_runs_are_bit_identical(env):
    torch, tm = env
    cfg = SMALL_LLAMA
    flat = si.make_flat_params(cfg)
    x, dy = to_dev(torch, si.make_x(cfg), cfg.dtype), to_dev(torch, si.make_dy(cfg), cfg.dtype)
    outs = []
    for _ in range(2):
        st = GpuStage(torch, tm, cfg, flat)
        st.fwd(x)
        st.bwd(dy)
        st.adam(step=1)
        torch.cuda.synchronize()
        outs.append((st.y.clone(), st.dx.clone(), st.grads.clone(), st.master.clone(), st.params.clone()))
        st.close()
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_state_overwritten_between_calls_is_used(env):
    """After the warm-up all local state is overwritten by the leaver's: the library must read the
    buffers at launch time and keep no copies."""
    torch, tm = env
    cfg = SMALL_GPT
    flat_a, flat_b = si.make_flat_params(cfg, seed=1), si.make_flat_params(cfg, seed=2)
    x = to_dev(torch, si.make_x(cfg), cfg.dtype)
    st = GpuStage(torch, tm, cfg, flat_a)
    ya = st.fwd(x).clone()
    st.params.copy_(to_dev(torch, flat_b, cfg.dtype))       # the "leaver's" parameters arrive
    yb = st.fwd(x).clone()
    ref = GpuStage(torch, tm, cfg, flat_b)
    yref = ref.fwd(x).clone()
    torch.cuda.synchronize()
    assert not torch.equal(ya, yb)
    assert torch.equal(yb, yref)
    st.close()
    ref.close()


def test_init_rejects_bad_buffers_and_shapes(env):
    torch, tm = env
    cfg = SMALL_GPT
    n = tm.tm_stage_param_count(cfg)
    buf = torch.zeros(n + 64, dtype=torch.float32, device="cuda")
    ws = torch.empty(tm.tm_stage_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    with pytest.raises(tm.TmError) as e:
        tm.tm_stage_init(cfg, buf, None, buf, buf, buf, ws)            # bf16 stage without master weights
    assert e.value.code == tm.TM_EINVAL
    with pytest.raises(tm.TmError) as e:
        tm.tm_stage_init(cfg, buf.data_ptr() + 4, buf, buf, buf, buf, ws)
    assert e.value.code == tm.TM_EALIGN
    with pytest.raises(tm.TmError) as e:
        tm.tm_stage_init(cfg.replace(n_q_heads=3), buf, buf, buf, buf, buf, ws)
    assert e.value.code == tm.TM_ESIZE
    with pytest.raises(tm.TmError) as e:                               # a workspace one byte short
        tm.tm_stage_init(cfg, buf, buf, buf, buf, buf, ws, workspace_bytes=ws.numel() - 1)
    assert e.value.code == tm.TM_ESIZE
