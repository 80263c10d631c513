"""The stage under the record / replay hook (sections 4.2, 4.3 of the paper), through the C ABI, against the CPU
checker's hooked stage: what a recording run stores, what a replaying run computes from a tape of seeded peer
tensors, boundary-only loading, and the error paths."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import sandbox_oracle as sb
from tests import tape_io
from tests.gpu_util import TOL_BF16, TOL_FP32, rel_err, require_gpu, stream_ptr, to_dev, to_host
from tests.stage_runner import GpuStage, flatten_grads

pytestmark = pytest.mark.gpu

SMALL_GPT = si.StageConfig(2, 256, 2, 2, 128, 512, 200, 2)
SMALL_LLAMA = si.StageConfig(2, 256, 4, 1, 64, 328, 130, 1, norm=si.NORM_RMSNORM, act=si.ACT_SWIGLU, pos=si.POS_ROTARY, has_bias=0)
TINY = si.PRESETS["tiny"]
ALL = sb.SCOPE_TP | sb.SCOPE_PP | sb.SCOPE_DP


@pytest.fixture(scope="module")
def env():
    torch = require_gpu()
    import paper_2412_12636_amd as tm
    assert (tm.TM_SCOPE_TP, tm.TM_SCOPE_PP, tm.TM_SCOPE_DP) == (sb.SCOPE_TP, sb.SCOPE_PP, sb.SCOPE_DP)
    assert (tm.TM_COLL_ALL_REDUCE, tm.TM_COLL_RECV, tm.TM_COLL_SEND, tm.TM_COLL_BARRIER) == (sb.ALL_REDUCE, sb.RECV, sb.SEND, sb.BARRIER)
    return torch, tm


def tol_of(cfg):
    return TOL_BF16 if cfg.dtype == si.DTYPE_BF16 else TOL_FP32


def gpu_iteration(torch, tm, cfg, st, comm, x, dy):
    """fwd, bwd, gradient sync under `comm`; returns host copies of y, dx and the flat gradients."""
    tm.tm_stage_attach_comm(st.handle, comm)
    tm.tm_stage_grad_mode(st.handle, True)
    y = to_host(st.fwd(to_dev(torch, x, cfg.dtype)))
    dx = to_host(st.bwd(to_dev(torch, dy, cfg.dtype)))
    tm.tm_stage_grad_sync(st.handle, stream_ptr(torch))
    torch.cuda.synchronize()
    tm.tm_stage_attach_comm(st.handle, None)
    return y, dx, st.grads.cpu().numpy().astype(np.float64)


def checker_iteration(cfg, layers, comm, x, dy):
    y, stashes = sb.stage_fwd(cfg, layers, x, comm)
    dx, grads = sb.stage_bwd(cfg, layers, stashes, dy, comm)
    return y, dx, sb.grad_sync(flatten_grads(cfg, grads), comm)


@pytest.mark.parametrize("cfg", [TINY, SMALL_GPT, SMALL_LLAMA], ids=["tiny_fp32", "small_gpt", "small_llama"])
def test_recording_run_stores_what_the_checker_stores(env, cfg, tmp_path):
    torch, tm = env
    print(f"record parity {cfg}", flush=True)
    flat, x, dy = si.make_flat_params(cfg), si.make_x(cfg), si.make_dy(cfg)
    layers = si.split_flat(cfg, flat)
    path = str(tmp_path / "rec.tape")
    st = GpuStage(torch, tm, cfg, flat)
    comm = tm.tm_comm_open(path, tm.TM_COMM_RECORD, ALL)
    y, dx, g = gpu_iteration(torch, tm, cfg, st, comm, x, dy)
    stats = tm.tm_comm_stats(comm)
    tm.tm_comm_close(comm)
    rec = sb.Recorder(sb.PassThrough(), ALL)
    ry, rdx, rg = checker_iteration(cfg, layers, rec, x, dy)
    tape = tape_io.read_tape(path)                        # verifies every checksum with the stated formula
    L = cfg.n_layers
    assert len(tape) == len(rec.tape) == 3 + 4 * L and stats["stored"] == len(tape)
    assert stats["calls"] == len(tape) + 3 and stats["native"] == 3     # two sends and the barrier
    tol = tol_of(cfg)
    for i, ((kind, scope, site, dtype, payload), (rk, rs, rsite, rdata)) in enumerate(zip(tape, rec.tape)):
        assert (kind, scope, site) == (rk, rs, rsite), i
        want_dtype = si.DTYPE_FP32 if site == sb.SITE_GRADS else cfg.dtype
        assert dtype == want_dtype and len(payload) == rdata.size * (2 if dtype == si.DTYPE_BF16 else 4)
        e = rel_err(tape_io.array_of(payload, dtype), rdata)
        assert e <= tol, (i, site, e)
    # with every call native the results are the plain stage's
    assert rel_err(y, ry) <= tol and rel_err(dx, rdx) <= tol and rel_err(g, rg) <= tol
    # what was stored for the pipeline receive is the argument itself, bit for bit
    assert tape[0][4] == tape_io.payload_of(x, cfg.dtype)
    st.close()


def peer_tape(cfg, scopes):
    """Seeded stand-ins for what recording ranks with real peers would have stored, in the stage's call order, with
    the magnitudes of the tensors they replace."""
    shape = (cfg.seq, cfg.micro_batch, cfg.hidden)
    snap = (lambda a: si.snap_to_bf16_grid(a)) if cfg.dtype == si.DTYPE_BF16 else (lambda a: a)
    draw = lambda i, site, std, shp=shape: snap(si.normal(si.BASE_SEED + 1, i, f"tape{site}", shp, std))
    out = [(sb.RECV, sb.SCOPE_PP, sb.SITE_X, draw(0, sb.SITE_X, 1.0))]
    for l in range(cfg.n_layers):
        out.append((sb.ALL_REDUCE, sb.SCOPE_TP, sb.SITE_ATTN_OUT, draw(l, sb.SITE_ATTN_OUT, 0.3)))
        out.append((sb.ALL_REDUCE, sb.SCOPE_TP, sb.SITE_MLP_OUT, draw(l, sb.SITE_MLP_OUT, 0.3)))
    out.append((sb.RECV, sb.SCOPE_PP, sb.SITE_DY, draw(0, sb.SITE_DY, 1e-2)))
    for l in reversed(range(cfg.n_layers)):
        out.append((sb.ALL_REDUCE, sb.SCOPE_TP, sb.SITE_D_MLP_IN, draw(l, sb.SITE_D_MLP_IN, 1e-2)))
        out.append((sb.ALL_REDUCE, sb.SCOPE_TP, sb.SITE_D_ATTN_IN, draw(l, sb.SITE_D_ATTN_IN, 1e-2)))
    out.append((sb.ALL_REDUCE, sb.SCOPE_DP, sb.SITE_GRADS, si.normal(si.BASE_SEED + 1, 0, "tapegrads", (si.stage_param_count(cfg),), 1e-3)))
    return [e for e in out if e[1] & scopes]


def write_peer_tape(path, cfg, entries):
    tape_io.write_tape(path, [(k, sc, site, si.DTYPE_FP32 if site == sb.SITE_GRADS else cfg.dtype,
                               tape_io.payload_of(a, si.DTYPE_FP32 if site == sb.SITE_GRADS else cfg.dtype))
                              for k, sc, site, a in entries])


@pytest.mark.parametrize("cfg", [TINY, SMALL_GPT, SMALL_LLAMA], ids=["tiny_fp32", "small_gpt", "small_llama"])
@pytest.mark.parametrize("boundary", [ALL, sb.SCOPE_PP, sb.SCOPE_PP | sb.SCOPE_DP, sb.SCOPE_TP], ids=["all", "pp", "pp_dp", "tp"])
def test_replaying_run_computes_what_the_checker_computes_from_the_same_tape(env, cfg, boundary, tmp_path):
    torch, tm = env
    print(f"replay parity boundary={boundary} {cfg}", flush=True)
    flat, x, dy = si.make_flat_params(cfg), si.make_x(cfg), si.make_dy(cfg)
    layers = si.split_flat(cfg, flat)
    entries = peer_tape(cfg, ALL)                       # the tape holds every scope; the boundary picks
    path = str(tmp_path / "peer.tape")
    write_peer_tape(path, cfg, entries)
    st = GpuStage(torch, tm, cfg, flat)
    comm = tm.tm_comm_open(path, tm.TM_COMM_REPLAY, boundary)
    on_boundary = [e for e in entries if e[1] & boundary]
    stats0 = tm.tm_comm_stats(comm)
    assert stats0["tape_entries"] == len(on_boundary)
    assert stats0["tape_bytes"] == sum(e[3].size * (4 if e[2] == sb.SITE_GRADS or cfg.dtype == si.DTYPE_FP32 else 2) for e in on_boundary)
    y, dx, g = gpu_iteration(torch, tm, cfg, st, comm, x, dy)
    stats = tm.tm_comm_stats(comm)
    rp = sb.Replayer([(k, sc, site, np.asarray(a, np.float64)) for k, sc, site, a in entries], boundary)
    ry, rdx, rg = checker_iteration(cfg, layers, rp, x, dy)
    tol = tol_of(cfg)
    errs = {"y": rel_err(y, ry), "dx": rel_err(dx, rdx), "grads": rel_err(g, rg)}
    print(f"  {errs}", flush=True)
    assert max(errs.values()) <= tol, errs
    assert stats["stored"] == rp.at == len(on_boundary) and stats["skipped"] == rp.skipped
    if boundary & sb.SCOPE_DP:                           # the reduced gradient is the tape's, bit for bit
        assert (g == entries[-1][3].astype(np.float64)).all()
    if boundary & sb.SCOPE_PP:                           # the arguments are ignored: other arguments, same results
        tm.tm_comm_rewind(comm)
        y2, dx2, g2 = gpu_iteration(torch, tm, cfg, st, comm, np.zeros_like(x), np.zeros_like(dy))
        assert (y2 == y).all() and (dx2 == dx).all() and (g2 == g).all()
    else:                                                # and a second shadow iteration repeats the first
        tm.tm_comm_rewind(comm)
        y2, dx2, g2 = gpu_iteration(torch, tm, cfg, st, comm, x, dy)
        assert (y2 == y).all() and (dx2 == dx).all() and (g2 == g).all()
    tm.tm_comm_close(comm)
    st.close()


def test_pass_through_hook_and_no_hook_give_the_same_bits(env):
    torch, tm = env
    cfg = SMALL_GPT
    flat, x, dy = si.make_flat_params(cfg), si.make_x(cfg), si.make_dy(cfg)
    st = GpuStage(torch, tm, cfg, flat)
    tm.tm_stage_grad_mode(st.handle, True)
    y0 = st.fwd(to_dev(torch, x, cfg.dtype)).clone()
    dx0 = st.bwd(to_dev(torch, dy, cfg.dtype)).clone()
    g0 = st.grads.clone()
    comm = tm.tm_comm_open(None, tm.TM_COMM_PASS, ALL)
    y, dx, g = gpu_iteration(torch, tm, cfg, st, comm, x, dy)
    assert (to_host(y0) == y).all() and (to_host(dx0) == dx).all() and (g0.cpu().numpy() == g).all()
    s = tm.tm_comm_stats(comm)
    assert s["calls"] == s["native"] == 6 + 4 * cfg.n_layers
    tm.tm_comm_close(comm)
    st.close()


def test_replay_error_paths(env, tmp_path):
    torch, tm = env
    cfg = TINY
    flat, x, dy = si.make_flat_params(cfg), si.make_x(cfg), si.make_dy(cfg)
    entries = peer_tape(cfg, ALL)
    path = str(tmp_path / "peer.tape")
    write_peer_tape(path, cfg, entries)
    st = GpuStage(torch, tm, cfg, flat)
    xd, dyd = to_dev(torch, x, cfg.dtype), to_dev(torch, dy, cfg.dtype)
    # backward first: the tape's next entry is the forward receive
    comm = tm.tm_comm_open(path, tm.TM_COMM_REPLAY, sb.SCOPE_PP)
    st.fwd(xd)
    tm.tm_stage_attach_comm(st.handle, comm)
    with pytest.raises(tm.TmError) as e:
        st.bwd(dyd)
    assert e.value.code == tm.TM_ESTATE
    # a second forward pass after the tape's two pipeline entries are used up
    tm.tm_comm_rewind(comm)
    st.fwd(xd)
    st.bwd(dyd)
    with pytest.raises(tm.TmError) as e:
        st.fwd(xd)
    assert e.value.code == tm.TM_ESTATE and "no entry left" in e.value.message
    torch.cuda.synchronize()
    tm.tm_stage_attach_comm(st.handle, None)
    tm.tm_comm_close(comm)
    # the fused backward + Adam call must not run ahead of an intercepted gradient reduction
    comm = tm.tm_comm_open(path, tm.TM_COMM_REPLAY, sb.SCOPE_DP)
    tm.tm_stage_attach_comm(st.handle, comm)
    st.fwd(xd)
    with pytest.raises(tm.TmError) as e:
        tm.tm_stage_bwd_adam(st.handle, dyd, st.dx, tm.make_hparams(**si.ADAM_DEFAULTS), 1, stream_ptr(torch))
    assert e.value.code == tm.TM_ESTATE
    tm.tm_stage_attach_comm(st.handle, None)
    tm.tm_comm_close(comm)
    # another stage shape: byte counts differ from the tape's
    other = cfg.replace(seq=cfg.seq // 2)
    st2 = GpuStage(torch, tm, other, si.make_flat_params(other))
    comm = tm.tm_comm_open(path, tm.TM_COMM_REPLAY, sb.SCOPE_PP)
    tm.tm_stage_attach_comm(st2.handle, comm)
    with pytest.raises(tm.TmError) as e:
        st2.fwd(to_dev(torch, si.make_x(other), other.dtype))
    assert e.value.code == tm.TM_ESTATE and "bytes" in e.value.message
    tm.tm_stage_attach_comm(st2.handle, None)
    tm.tm_comm_close(comm)
    # a flipped payload bit fails the checksum at open
    raw = bytearray(open(path, "rb").read())
    raw[16 + 64 + 5] ^= 0x10
    bad = str(tmp_path / "bad.tape")
    open(bad, "wb").write(bytes(raw))
    with pytest.raises(tm.TmError) as e:
        tm.tm_comm_open(bad, tm.TM_COMM_REPLAY, sb.SCOPE_PP)
    assert e.value.code == tm.TM_ESTATE and "checksum" in e.value.message
    torch.cuda.synchronize()
    st.close()
    st2.close()


@pytest.mark.parametrize("dtype", [si.DTYPE_BF16, si.DTYPE_FP32])
@pytest.mark.parametrize("T,h,bias", [(37, 264, True), (5, 8, False), (300, 1024, True)])
def test_bias_residual_add(env, dtype, T, h, bias):
    torch, tm = env
    rng = np.random.default_rng(3)
    snap = (lambda a: si.snap_to_bf16_grid(a.astype(np.float32))) if dtype == si.DTYPE_BF16 else (lambda a: a.astype(np.float32))
    part, res, b = snap(rng.standard_normal((T, h))), snap(rng.standard_normal((T, h))), snap(rng.standard_normal(h) * 0.1)
    out = torch.empty((T, h), dtype=torch.bfloat16 if dtype == si.DTYPE_BF16 else torch.float32, device="cuda")
    tm.tm_op_bias_residual_add(dtype, T, h, to_dev(torch, part, dtype), to_dev(torch, b, dtype) if bias else None,
                               to_dev(torch, res, dtype), out, stream_ptr(torch))
    torch.cuda.synchronize()
    want = part.astype(np.float64) + res + (b if bias else 0.0)
    assert rel_err(to_host(out), want) <= (4e-3 if dtype == si.DTYPE_BF16 else 1e-6)
