#!/usr/bin/env python3
"""Throughput of the stage-shard iteration (forward + backward + Adam) on one MI355X.

A step is one pass of the whole hot path over one synthetic micro-batch of the chosen shard
preset: tm_stage_fwd, then tm_stage_bwd_adam (backward pass with the Adam update; gradients transient).
Inputs and all state are resident in HBM before the timed region.  One JSON line is printed.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--preset gpt175b] [--cpu-seconds 20]

Timing: W untimed steps, then K steps bracketed by device synchronisation and HIP events on the
stream the kernels are launched on.  The same work as three separate calls (forward, backward, Adam) is
timed next: its forward + backward time gives the matrix-core utilisation.  A third pass repeats the TIMED
form of the step with the library's per-kernel event profiling switched on (same kernels, same stream, every
launch bracketed by two events); the kernel with the largest total time gives the `roofline` object
(algorithmic flops or bytes of its launches / their summed duration).  The CPU checker is timed on
a bounded sample of the same workload for `cpu_baseline`.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def recorded_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None when
    there is none or the kernel's source has changed since the counters were taken."""
    import glob
    import hashlib
    import re
    for path in glob.glob(os.path.join(ROOT, "profiles", "*traffic*.txt")):
        text = open(path).read()
        m = re.search(r"^kernel:\s*(.+?)\s*$", text, re.M)
        if not m or kernel != m.group(1):
            continue
        src = re.search(r"^source:\s*(\S+)\s+sha256:\s*([0-9a-f]+)", text, re.M)
        val = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
        if not src or not val:
            continue
        cur = hashlib.sha256(open(os.path.join(ROOT, src.group(1)), "rb").read()).hexdigest()
        return float(val.group(1)) if cur == src.group(2) else None
    return None


def model_flops(cfg) -> float:
    """Model flops of one iteration: 3 x forward; attention counted causal (half the square), no
    credit for recomputation."""
    T = cfg.seq * cfg.micro_batch
    gemm = 2.0 * T * (cfg.qkv_width * cfg.hidden + cfg.hidden * cfg.attn_width + cfg.fc1_width * cfg.hidden
                      + cfg.hidden * cfg.ffn)
    attn = 2.0 * cfg.micro_batch * cfg.n_q_heads * cfg.seq * cfg.seq * cfg.head_dim
    return 3.0 * cfg.n_layers * (gemm + attn)


def cpu_baseline(si, cfg, preset: str, budget_s: float):
    """Times the fp64 CPU checker (forward, backward, Adam; best of 3) and scales to the whole stage.  The small
    presets run whole (all layers, all positions) and get a 1-thread figure beside the all-cores one; the large
    ones run one layer at a reduced token count: forward/backward time is linear in tokens (attention is a small
    share) and in layers, Adam is per parameter.  Returns the dict for the JSON line."""
    import numpy as np
    from oracle import stage_oracle as so
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        threadpool_limits = None
        threads = len(os.sched_getaffinity(0))
    whole = si.stage_param_count(cfg) <= 150_000_000
    seq_s = cfg.seq if whole else min(cfg.seq, 512)
    n_l = cfg.n_layers if whole else 1
    sample = cfg.replace(n_layers=n_l, seq=seq_s)
    layers = [si.make_layer_params(sample, l) for l in range(n_l)]
    x, dy = si.make_x(sample), si.make_dy(sample)

    def once():
        t0 = time.time()
        y, st = so.stage_fwd(sample, layers, x)
        dx, gr = so.stage_bwd(sample, layers, st, dy)
        t_fb = time.time() - t0
        # Adam on the first layer's largest matrix, scaled to the sample's parameter count
        name = max(gr[0], key=lambda k: gr[0][k].size)
        w = layers[0][name].astype(np.float64)
        z = np.zeros_like(w)
        t0 = time.time()
        w2, m2, v2 = so.adam_step(w, gr[0][name], z, z, 1, 1e-3, 0.9, 0.999, 1e-8)
        so.bf16_round_nearest_even(w2.astype(np.float32))
        t_adam = (time.time() - t0) * si.stage_param_count(sample) / w.size
        return t_fb, t_adam

    t_start = time.time()
    runs = []
    for _ in range(3):
        runs.append(once())
        if time.time() - t_start > 2.0 * budget_s:      # a slow host: what has been measured stands
            break
    t_fb, t_adam = min(runs, key=lambda r: r[0] + r[1])
    scale_l, scale_t = cfg.n_layers / n_l, cfg.seq / seq_s
    step_s = scale_l * (t_fb * scale_t + t_adam)
    try:
        cpu_model = next(l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name"))
    except Exception:
        cpu_model = "unknown"
    out = {
        "value": cfg.seq * cfg.micro_batch / step_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"fp64 numpy checker, best of {len(runs)}: {n_l} of {cfg.n_layers} layers at full width, first {seq_s} of "
                   f"{cfg.seq} positions: fwd+bwd {t_fb:.2f} s, Adam {t_adam:.2f} s"
                   + ("" if whole else f"; extrapolated x{cfg.seq // seq_s} in tokens (Adam not) and x{cfg.n_layers} in layers")),
        "measured_s": round(t_fb + t_adam, 2), "runs_s": [round(a + b, 2) for a, b in runs],
        "host_cpus": len(os.sched_getaffinity(0)), "blas_threads": int(threads), "cpu_model": cpu_model,
        "fp64_gflops": round(model_flops(sample) / t_fb / 1e9, 1), "extrapolated": not whole,
    }
    if whole and threadpool_limits is not None:
        with threadpool_limits(limits=1):
            t1_fb, t1_adam = once()
        out["one_thread"] = {"value": cfg.seq * cfg.micro_batch / (t1_fb + t1_adam), "unit": "tokens/s",
                             "fwd_bwd_s": round(t1_fb, 2), "adam_s": round(t1_adam, 2)}
    return out


def time_sandbox(torch, tm, h, x, y, dy, dx, stream: int, folder: str, reps: int):
    """Forward + backward of one micro-batch with the hook attached: a recording run (synchronous by design: every stored
    tensor is complete before it goes to the tape), the tape's load into pinned host memory, and replaying runs."""
    os.makedirs(folder, exist_ok=True)

    def fwd_bwd():
        tm.tm_stage_fwd(h, x, y, stream)
        tm.tm_stage_bwd(h, dy, dx, stream)

    def wall(fn, n):
        torch.cuda.synchronize()
        t0 = time.time()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.time() - t0) * 1e3 / n

    fwd_bwd()
    res = {"plain_ms": round(wall(fwd_bwd, reps), 3)}
    for label, scopes in (("pp", tm.TM_SCOPE_PP), ("pp_tp", tm.TM_SCOPE_PP | tm.TM_SCOPE_TP)):
        path = os.path.join(folder, f"bench_{label}.tape")
        c = tm.tm_comm_open(path, tm.TM_COMM_RECORD, scopes)
        tm.tm_stage_attach_comm(h, c)
        rec_ms = wall(fwd_bwd, 1)
        st = tm.tm_comm_stats(c)
        tm.tm_stage_attach_comm(h, None)
        tm.tm_comm_close(c)
        t0 = time.time()
        c = tm.tm_comm_open(path, tm.TM_COMM_REPLAY, scopes)
        load_s = time.time() - t0
        tm.tm_stage_attach_comm(h, c)

        def replay():
            tm.tm_comm_rewind(c)
            fwd_bwd()

        replay()
        rep_ms = wall(replay, reps)
        tm.tm_stage_attach_comm(h, None)
        torch.cuda.synchronize()
        tm.tm_comm_close(c)
        os.remove(path)
        res[label] = {"tape_entries": st["stored"], "tape_bytes": st["stored_bytes"], "record_ms": round(rec_ms, 3),
                      "tape_load_s": round(load_s, 3), "tape_load_gbps": round(st["stored_bytes"] / max(load_s, 1e-9) / 1e9, 2),
                      "replay_ms": round(rep_ms, 3)}
    res["note"] = ("host wall clock per forward + backward; replay enqueues one host-to-device copy per boundary tensor; with "
                   "the tensor scope intercepted the two row-parallel products run without their fused bias/residual epilogue")
    return res


def time_moe(torch, tm, si, gen, stream: int, reps: int):
    """tm_moe_fwd, tm_moe_bwd (gradients stored, not added) and the flat Adam sweep over the shard's parameters."""
    cfg = si.MOE_PRESETS["moe5t"]
    n = tm.tm_moe_param_count(cfg)
    master = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=gen)
    params = master.to(torch.bfloat16)
    master.copy_(params)
    grads, m, v = (torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(3))
    c = torch.empty((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda").normal_(0, 1, generator=gen).to(torch.bfloat16)
    dout = torch.empty((cfg.tokens, cfg.hidden), dtype=torch.float32, device="cuda").normal_(0, 1e-2, generator=gen).to(torch.bfloat16)
    out, dc = torch.empty_like(c), torch.empty_like(c)
    ws = torch.empty(tm.tm_moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    hp = tm.make_hparams(**si.ADAM_DEFAULTS)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    tot = [0.0, 0.0, 0.0]
    for it in range(reps + 2):
        ev[0].record()
        tm.tm_moe_fwd(cfg, params, c, out, ws, stream)
        ev[1].record()
        tm.tm_moe_bwd(cfg, params, c, dout, dc, grads, 0, ws, stream)
        ev[2].record()
        tm.tm_adam_step_flat(n, master, grads, m, v, params, hp, it + 1, stream)
        ev[3].record()
        torch.cuda.synchronize()
        if it >= 2:
            for i in range(3):
                tot[i] += ev[i].elapsed_time(ev[i + 1])
    fwd, bwd, adam = (t / reps for t in tot)
    rows = cfg.n_experts * cfg.capacity
    flops = 3 * (2.0 * rows * cfg.hidden * cfg.ffn * 2 + 2.0 * cfg.tokens * cfg.n_experts * cfg.hidden)
    return {"workload": f"moe5t: {cfg.tokens} tokens, hidden {cfg.hidden}, expert width {cfg.ffn}, {cfg.n_experts} experts over "
                        f"ep {cfg.ep}, top-{cfg.top_k}, capacity {cfg.capacity} rows per expert buffer, {n} parameters",
            "fwd_ms": round(fwd, 3), "bwd_ms": round(bwd, 3), "adam_ms": round(adam, 3),
            "tokens_per_s": round(cfg.tokens / ((fwd + bwd + adam) * 1e-3), 1),
            "tflops_fwd_bwd": round(flops / ((fwd + bwd) * 1e-3) / 1e12, 1),
            "mfma_frac_fwd_bwd": round(flops / ((fwd + bwd) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "adam_gbps": round(30.0 * n / (adam * 1e-3) / 1e9, 1),
            "note": "model flops: 3 x (two expert products over all buffer rows + the router product)"}


def time_roles(torch, tm, cfg, v_local: int, gen, stream: int, reps: int):
    """The layers only the first and the last pipeline stage have, at the preset's width: embedding lookup and its
    scatter-add backward; final norm + output layer + cross-entropy over the shard, forward and backward in one call."""
    seq, batch, h = cfg.seq, cfg.micro_batch, cfg.hidden
    T, v0 = seq * batch, 2 * v_local
    td = torch.bfloat16

    def draw(shape, std, mean=0.0):
        return torch.empty(shape, dtype=torch.float32, device="cuda").normal_(mean, std, generator=gen).to(td)

    w, pos, y, dx0 = draw((v_local, h), 0.02), draw((seq, h), 0.02), draw((seq, batch, h), 1.0), draw((seq, batch, h), 0.01)
    gain, offset = draw((h,), 0.02, 1.0), draw((h,), 0.02)
    tokens = torch.randint(0, 8 * v_local, (T,), generator=gen, device="cuda", dtype=torch.int32)
    tokens[:T // 2] = torch.randint(v0, v0 + v_local, (T // 2,), generator=gen, device="cuda", dtype=torch.int32)
    x0, dy = torch.empty_like(y), torch.empty_like(y)
    dw = torch.empty((v_local, h), dtype=torch.float32, device="cuda")
    dpos = torch.empty((seq, h), dtype=torch.float32, device="cuda")
    dgain, doffset = (torch.empty(h, dtype=torch.float32, device="cuda") for _ in range(2))
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(tm.tm_head_workspace_bytes(1, seq, batch, h, v_local), dtype=torch.uint8, device="cuda")
    ln = cfg.norm == 0

    def timed(fn):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_ef = timed(lambda: tm.tm_op_embed_fwd(1, seq, batch, h, v_local, v0, tokens, w, pos, x0, stream))
    t_eb = timed(lambda: tm.tm_op_embed_bwd(1, seq, batch, h, v_local, v0, tokens, dx0, dw, dpos, seq, 0, stream))
    t_head = timed(lambda: tm.tm_head_fwd_bwd(1, cfg.norm, cfg.norm_eps, seq, batch, h, v_local, v0, y, tokens, gain,
                                              offset if ln else None, w, 1.0, ws, loss, dy, dgain, doffset if ln else None,
                                              dw, 0, stream))
    head_flops = 3 * 2.0 * T * v_local * h
    return {"v_local": v_local, "tokens": T, "hidden": h,
            "embed_fwd_ms": round(t_ef, 4), "embed_fwd_gbps": round((T * h * 2 * 3) / (t_ef * 1e-3) / 1e9, 1),
            "embed_bwd_ms": round(t_eb, 4), "embed_bwd_gbps": round((T * h * 2 + (v_local + seq) * h * 4) / (t_eb * 1e-3) / 1e9, 1),
            "head_fwd_bwd_ms": round(t_head, 4), "head_tflops": round(head_flops / (t_head * 1e-3) / 1e12, 1),
            "note": "bytes: embedding forward reads a table row and a position row and writes x0 per token; backward reads "
                    "dx0 once and writes both fp32 gradients once; head flops = 3 products of 2*T*v_local*h"}


def power_probe(torch, tm, cfg, gen, stream: int, reps: int = 300):
    """The largest forward product of the preset (FC1), sustained over `reps` back-to-back launches that rotate
    through twelve weight matrices, once with the recipe's random operands and once with all-zero operands: the same
    kernel, the same memory traffic and instruction stream, only the switching activity of the data differs.  A large
    gap says the matrix cores run against the chip's power limit, not against issue or memory limits."""
    T, N, K, nl = cfg.seq * cfg.micro_batch, cfg.fc1_width, cfg.hidden, 12
    out = {"shape": [T, N, K], "reps": reps}
    y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    for kind in ("random", "zeros"):
        if kind == "random":
            x = torch.empty((T, K), dtype=torch.float32, device="cuda").normal_(0, 1, generator=gen).to(torch.bfloat16)
            w = torch.empty((nl, N, K), dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=gen).to(torch.bfloat16)
        else:
            x = torch.zeros((T, K), dtype=torch.bfloat16, device="cuda")
            w = torch.zeros((nl, N, K), dtype=torch.bfloat16, device="cuda")
        for r in range(20):
            tm.tm_op_linear_fwd(1, T, N, K, x, w[r % nl], None, None, y, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for r in range(reps):
            tm.tm_op_linear_fwd(1, T, N, K, x, w[r % nl], None, None, y, stream)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[kind] = {"ms": round(ms, 5), "tflops": round(2.0 * T * N * K / (ms * 1e-3) / 1e12, 1)}
        del x, w
    out["zeros_over_random"] = round(out["zeros"]["tflops"] / out["random"]["tflops"], 4)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--preset", default="gpt175b")
    ap.add_argument("--layers", type=int, default=0, help="override the preset's layer count (0 = preset)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 4 GiB device copy before the timed region (reference reading "
                         "for the FETCH_SIZE / WRITE_SIZE counters under rocprofv3 --pmc)")
    ap.add_argument("--micro-batches", type=int, default=12,
                    help="also time a whole iteration of this many micro-batches (gradient accumulation, squared "
                         "gradient norm, clipping factor on the host, Adam on one data-parallel rank's slice); the paper's "
                         "default profiles run 12 to 16 per iteration; 0 leaves it out")
    ap.add_argument("--dp", type=int, default=3, help="data-parallel size for --micro-batches (Adam updates 1/dp)")
    ap.add_argument("--clip", type=float, default=1.0, help="gradient-norm limit for --micro-batches (0: off)")
    ap.add_argument("--sandbox", default="", metavar="DIR",
                    help="also time the shadow iteration (forward + backward, one micro-batch) under the record / replay "
                         "hook, tapes written to DIR: recording and replaying the pipeline scope, and pipeline + tensor scope")
    ap.add_argument("--moe", action="store_true",
                    help="also time forward + backward + Adam of the mixture-of-experts MLP shard shaped like the paper's "
                         "5.12T-parameter workload (one local expert, 16 experts, top-2, 2048 tokens)")
    ap.add_argument("--power-probe", action="store_true",
                    help="also time the preset's FC1 forward product sustained, with random and with all-zero operands "
                         "(same kernel and traffic; the gap shows how far the matrix cores run against the power limit)")
    ap.add_argument("--roles", type=int, default=0, metavar="V_LOCAL",
                    help="also time the first- and last-stage layers at the preset's width with this many vocabulary "
                         "rows per rank (e.g. 6400 = 51200 / 8)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's stage shard; this build has no multi-GPU path "
              "(collectives are identities by design). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2412_12636_amd as tm
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    cfg = si.PRESETS[args.preset]
    if args.layers:
        cfg = cfg.replace(n_layers=args.layers)
    bf16 = cfg.dtype == si.DTYPE_BF16
    td = torch.bfloat16 if bf16 else torch.float32
    n = tm.tm_stage_param_count(cfg)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(si.BASE_SEED)

    # state, resident in HBM: N(0, 0.02^2) everywhere, norm gains shifted to 1
    master = torch.empty(n, dtype=torch.float32, device="cuda")
    chunk = 1 << 28
    for lo in range(0, n, chunk):
        master[lo:lo + chunk].normal_(0.0, 0.02, generator=gen)
    for name, off, shape in tm.tm_stage_param_layout(cfg):
        if name.endswith("_gain"):
            master[off:off + shape[0]] += 1.0
    params = master.to(td) if bf16 else master
    if bf16:
        master.copy_(params)          # master starts from the bf16-representable values
    grads = torch.zeros(n, dtype=torch.float32, device="cuda")
    m = torch.zeros(n, dtype=torch.float32, device="cuda")
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    ws = torch.empty(tm.tm_stage_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
    shape = (cfg.seq, cfg.micro_batch, cfg.hidden)
    x = torch.empty(shape, dtype=torch.float32, device="cuda").normal_(0, 1, generator=gen).to(td)
    dy = torch.empty(shape, dtype=torch.float32, device="cuda").normal_(0, 1e-2, generator=gen).to(td)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    h = tm.tm_stage_init(cfg, params, master if bf16 else None, grads, m, v, ws)
    # one micro-batch per iteration: the backward pass stores the gradients (their old contents are
    # dead), so nothing has to clear the buffer and Adam only reads it; in the timed step (backward with the
    # update) nobody reads the gradients afterwards, so the matrices' gradients may stay in registers
    tm.tm_stage_grad_mode(h, tm.TM_GRAD_TRANSIENT)
    # once per process: time the GEMM tile configurations on this shard's twelve products
    tm.tm_stage_tune(h, int(torch.cuda.current_stream().cuda_stream))
    hp = tm.make_hparams(**si.ADAM_DEFAULTS)
    stream = int(torch.cuda.current_stream().cuda_stream)
    step_no = [0]

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def one_step(marks=None):
        """The step as timed: forward, then backward with every layer's Adam update enqueued as soon as that
        layer's gradients are complete (same results as the three separate calls below)."""
        step_no[0] += 1
        if marks is not None:
            marks[0].record()
        tm.tm_stage_fwd(h, x, y, stream)
        if marks is not None:
            marks[1].record()
        tm.tm_stage_bwd_adam(h, dy, dx, hp, step_no[0], stream)
        if marks is not None:
            marks[2].record()

    def one_step_sequential(marks=None):
        step_no[0] += 1
        if marks is not None:
            marks[0].record()
        tm.tm_stage_fwd(h, x, y, stream)
        if marks is not None:
            marks[1].record()
        tm.tm_stage_bwd(h, dy, dx, stream)
        if marks is not None:
            marks[2].record()
        tm.tm_adam_step(h, hp, step_no[0], stream)
        if marks is not None:
            marks[3].record()

    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # cold first call (the gap the sandboxed warm-up exists to hide)
    torch.cuda.synchronize()
    t0 = time.time()
    one_step()
    torch.cuda.synchronize()
    first_ms = (time.time() - t0) * 1e3
    for _ in range(max(0, args.warmup - 1)):
        one_step()
    torch.cuda.synchronize()

    marks = [[ev() for _ in range(4)] for _ in range(args.steps)]
    start, stop = ev(), ev()
    torch.cuda.synchronize()
    t0 = time.time()
    start.record()
    for k in range(args.steps):
        one_step(marks[k])
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.time() - t0) * 1e3
    total_ms = start.elapsed_time(stop)
    ms_step = total_ms / args.steps
    fwd_ms = sum(mk[0].elapsed_time(mk[1]) for mk in marks) / args.steps
    bwd_adam_ms = sum(mk[1].elapsed_time(mk[2]) for mk in marks) / args.steps

    # the same work as three separate calls, for the per-phase figures
    sstart, sstop = ev(), ev()
    sstart.record()
    for k in range(args.steps):
        one_step_sequential(marks[k])
    sstop.record()
    torch.cuda.synchronize()
    seq_ms_step = sstart.elapsed_time(sstop) / args.steps
    seq_fwd_ms = sum(mk[0].elapsed_time(mk[1]) for mk in marks) / args.steps
    bwd_ms = sum(mk[1].elapsed_time(mk[2]) for mk in marks) / args.steps
    adam_ms = sum(mk[2].elapsed_time(mk[3]) for mk in marks) / args.steps

    def profiled(step_fn):
        """K steps with every launch bracketed by two events on the launch stream; per-kernel totals, largest first."""
        tm.tm_stage_profile_enable(h, True)
        torch.cuda.synchronize()
        p0, p1 = ev(), ev()
        p0.record()
        for _ in range(args.steps):
            step_fn()
        p1.record()
        torch.cuda.synchronize()
        rows = tm.tm_stage_profile_collect(h, 64)
        tm.tm_stage_profile_enable(h, False)
        rows.sort(key=lambda e: -e["ms"])
        return rows, p0.elapsed_time(p1) / args.steps

    def bound_of(e):
        """A kernel's roofline: the bound that needs the longer time at the chip's peak for the kernel's algorithmic
        work (a weight-gradient product that also applies the update has both flops and bytes)."""
        t_mfma, t_hbm = e["flops"] / (PEAK_BF16_TFLOPS * 1e12), e["bytes"] / (PEAK_HBM_GBS * 1e9)
        secs = e["ms"] * 1e-3
        r = {"kernel": e["kernel"], "avg_launch_ms": round(e["ms"] / e["launches"], 5), "launches": e["launches"]}
        if t_mfma >= t_hbm:
            ach = e["flops"] / secs / 1e12
            r.update({"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                      "frac": round(ach / PEAK_BF16_TFLOPS, 4)})
        else:
            ach = e["bytes"] / secs / 1e9
            r.update({"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                      "frac": round(ach / PEAK_HBM_GBS, 4)})
        if e["flops"] > 0 and e["bytes"] > 0:       # both kinds of work: say what the other one amounts to
            r["also"] = {"tflops": round(e["flops"] / secs / 1e12, 1), "gbps": round(e["bytes"] / secs / 1e9, 1),
                         "time_at_peaks_ms": {"mfma": round(t_mfma * 1e3 / e["launches"], 5), "hbm": round(t_hbm * 1e3 / e["launches"], 5)}}
        r["traffic"] = recorded_traffic(e["kernel"])
        return r

    def kernel_rows(rows):
        out_rows = []
        for e in rows:
            row = {"kernel": e["kernel"], "launches_per_step": e["launches"] // args.steps,
                   "ms_per_step": round(e["ms"] / args.steps, 4), "avg_launch_ms": round(e["ms"] / e["launches"], 5)}
            if e["flops"] > 0:
                row["tflops"] = round(e["flops"] / (e["ms"] * 1e-3) / 1e12, 1)
            if e["bytes"] > 0:
                row["gbps"] = round(e["bytes"] / (e["ms"] * 1e-3) / 1e9, 1)
            out_rows.append(row)
        return out_rows

    # third pass: the step AS TIMED (forward, backward with the update), per-kernel events on the launch stream
    prof, prof_ms_step = profiled(one_step)
    kernels = kernel_rows(prof)
    roofline = bound_of(prof[0])
    # the largest kernel that only multiplies (forward and input-gradient products carry no update)
    roofline_mfma = next((bound_of(e) for e in prof if e["flops"] > 0 and e["bytes"] == 0 and "gemm" in e["kernel"]), None)
    # fourth pass: the three-call form, for the plain weight-gradient product and the flat Adam sweep
    prof_seq, prof_seq_ms_step = profiled(one_step_sequential)
    roofline_hbm = next((bound_of(e) for e in prof_seq if e["kernel"] == "adam_kernel"), None)
    roofline_wgrad = next((bound_of(e) for e in prof_seq if "epi2" in e["kernel"] and "ks,ks" in e["kernel"]), None)

    tokens = cfg.seq * cfg.micro_batch
    flops = model_flops(cfg)
    tf = flops / ((seq_fwd_ms + bwd_ms) * 1e-3) / 1e12
    adam_bytes = (30.0 if bf16 else 28.0) * n
    out = {
        "metric": "stage-shard fwd+bwd+Adam tokens/s per GPU; MFMA util % of bf16 peak",
        "value": round(tokens / (ms_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.preset}: {cfg.n_layers} layers, hidden {cfg.hidden}, {cfg.n_q_heads}q/"
                               f"{cfg.n_kv_heads}kv heads x {cfg.head_dim}, ffn {cfg.ffn}, seq {cfg.seq}, "
                               f"micro-batch {cfg.micro_batch}, {n} parameters (one rank's TP shard of one PP stage)",
                   "preset": args.preset, "tokens_per_step": tokens},
        "step": "tm_stage_fwd + tm_stage_bwd_adam, transient gradients (each weight matrix is updated in the epilogue of its "
                "weight-gradient product from the accumulators, the vectors by a flat sweep beside the layers below; same "
                "bits as the three separate calls, which are timed as sequential_*)",
        "phases_ms": {"fwd": round(fwd_ms, 4), "bwd_with_adam": round(bwd_adam_ms, 4)},
        "sequential_ms_per_step": round(seq_ms_step, 4),
        "sequential_phases_ms": {"fwd": round(seq_fwd_ms, 4), "bwd": round(bwd_ms, 4), "adam": round(adam_ms, 4)},
        "tflops_fwd_bwd": round(tf, 2), "mfma_frac_fwd_bwd": round(tf / PEAK_BF16_TFLOPS, 4),
        "model_tflop_per_step": round(flops / 1e12, 3),
        "adam_gbps": round(adam_bytes / (adam_ms * 1e-3) / 1e9, 1), "adam_frac_hbm": round(adam_bytes / (adam_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        "first_step_ms": round(first_ms, 2), "host_wall_ms_per_step": round(wall_ms / args.steps, 4),
        "profiled_ms_per_step": round(prof_ms_step, 4), "profiled_sequential_ms_per_step": round(prof_seq_ms_step, 4),
        "roofline": roofline, "roofline_mfma": roofline_mfma, "roofline_hbm": roofline_hbm, "roofline_wgrad_unfused": roofline_wgrad,
        "kernels": kernels[:16], "kernels_sequential": kernel_rows(prof_seq)[:6],
    }
    if args.micro_batches > 0:
        # the iteration of the paper's default profiles (section 8.1): n micro-batches, one optimizer step on 1/dp
        nmb, dp = args.micro_batches, max(1, args.dp)
        share = -(-(-(-n // dp)) // 8) * 8
        first, count = 0, min(n, share)
        sq = torch.zeros(1, dtype=torch.float64, device="cuda")

        def iteration():
            step_no[0] += 1
            for i in range(nmb):
                tm.tm_stage_grad_mode(h, i == 0)
                tm.tm_stage_fwd(h, x, y, stream)
                tm.tm_stage_bwd(h, dy, dx, stream)
            tm.tm_stage_grad_sq_sum(h, sq, stream)
            norm = math.sqrt(float(sq.item())) / nmb          # the host waits here, as a training loop does
            factor = (1.0 / nmb) * (min(1.0, args.clip / (norm + 1e-6)) if args.clip > 0 else 1.0)
            tm.tm_adam_step_range(h, first, count, tm.make_hparams(**{**si.ADAM_DEFAULTS, "grad_scale": factor}),
                                  step_no[0], stream)

        iteration()
        torch.cuda.synchronize()
        n_it = max(1, min(3, args.steps // 3))
        t0 = time.time()
        for _ in range(n_it):
            iteration()
        torch.cuda.synchronize()
        it_ms = (time.time() - t0) * 1e3 / n_it
        out["iteration"] = {"micro_batches": nmb, "dp": dp, "clip": args.clip, "ms": round(it_ms, 3),
                            "tokens_per_s": round(nmb * tokens / (it_ms * 1e-3), 1),
                            "tflops_whole_iteration": round(nmb * flops / (it_ms * 1e-3) / 1e12, 1),
                            "mfma_frac_whole_iteration": round(nmb * flops / (it_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                            "iterations_timed": n_it,
                            "note": "host wall clock over whole iterations (forward, backward, gradient norm, host-side "
                                    "clipping factor, Adam on 1/dp of the state); gradient accumulation from the second micro-batch on"}
        tm.tm_stage_grad_mode(h, tm.TM_GRAD_TRANSIENT)
    if args.sandbox:
        out["sandbox"] = time_sandbox(torch, tm, h, x, y, dy, dx, stream, args.sandbox, max(3, args.steps))
    if args.moe:
        out["moe"] = time_moe(torch, tm, si, gen, stream, max(3, args.steps))
    if args.roles > 0:
        out["roles"] = time_roles(torch, tm, cfg, args.roles, gen, stream, max(3, args.steps))
    if args.power_probe:
        out["power_probe"] = power_probe(torch, tm, cfg, gen, stream)
    tm.tm_stage_destroy(h)
    if not args.no_cpu_baseline:
        del master, params, grads, m, v, ws
        out["cpu_baseline"] = cpu_baseline(si, cfg, args.preset, args.cpu_seconds)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
