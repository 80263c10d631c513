"""Runs one stage-shard iteration on the GPU through the C ABI and on the CPU checker, from the
same seeded inputs, and returns both sides for comparison."""
from __future__ import annotations

import time
from typing import Dict, List

import numpy as np

import synth_inputs as si
from oracle import stage_oracle as so
from tests.gpu_util import f32_dev, stream_ptr, to_dev, to_host, torch_dtype


class GpuStage:
    """Device buffers of one stage plus its handle."""

    def __init__(self, torch, tm, cfg: si.StageConfig, flat_params: np.ndarray):
        self.torch, self.tm, self.cfg = torch, tm, cfg
        n = tm.tm_stage_param_count(cfg)
        assert n == flat_params.size
        self.n = n
        self.params = to_dev(torch, flat_params, cfg.dtype)
        self.master = f32_dev(torch, flat_params) if cfg.dtype == si.DTYPE_BF16 else None
        self.grads = torch.zeros(n, dtype=torch.float32, device="cuda")
        self.m = torch.zeros(n, dtype=torch.float32, device="cuda")
        self.v = torch.zeros(n, dtype=torch.float32, device="cuda")
        self.workspace = torch.empty(tm.tm_stage_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
        self.handle = tm.tm_stage_init(cfg, self.params, self.master, self.grads, self.m, self.v, self.workspace)
        td = torch_dtype(torch, cfg.dtype)
        shape = (cfg.seq, cfg.micro_batch, cfg.hidden)
        self.y = torch.empty(shape, dtype=td, device="cuda")
        self.dx = torch.empty(shape, dtype=td, device="cuda")

    def fwd(self, x):
        self.tm.tm_stage_fwd(self.handle, x, self.y, stream_ptr(self.torch))
        return self.y

    def bwd(self, dy):
        self.tm.tm_stage_bwd(self.handle, dy, self.dx, stream_ptr(self.torch))
        return self.dx

    def adam(self, step=1, **kw):
        hp = self.tm.make_hparams(**{**si.ADAM_DEFAULTS, **kw})
        self.tm.tm_adam_step(self.handle, hp, step, stream_ptr(self.torch))

    def master_weights(self):
        return self.master if self.master is not None else self.params

    def close(self):
        self.tm.tm_stage_destroy(self.handle)
        self.handle = None


def oracle_iteration(cfg: si.StageConfig, layers: List[Dict[str, np.ndarray]], x: np.ndarray, dy: np.ndarray,
                     progress=False):
    """fp64 forward and backward through all layers.  Returns y, dx, list of gradient dicts.  progress: True prints
    each completed layer; a callable receives the line instead (the conftest fixture that bypasses capture)."""
    say = progress if callable(progress) else ((lambda m: print(m, flush=True)) if progress else (lambda m: None))
    t0 = time.time()
    stashes = []
    y = x
    for i, p in enumerate(layers):
        y, st = so.layer_fwd(cfg, p, y)
        stashes.append(st)
        say(f"  checker forward layer {i} done at {time.time() - t0:.1f} s")
    grads = [None] * len(layers)
    dx = dy
    for i in reversed(range(len(layers))):
        dx, grads[i] = so.layer_bwd(cfg, layers[i], stashes[i], dx)
        stashes[i] = None
        say(f"  checker backward layer {i} done at {time.time() - t0:.1f} s")
    return y, dx, grads


def flatten_grads(cfg: si.StageConfig, grads: List[Dict[str, np.ndarray]]) -> np.ndarray:
    out = np.empty(si.stage_param_count(cfg), dtype=np.float64)
    off = 0
    for g in grads:
        for name, shape in si.layer_inventory(cfg):
            n = int(np.prod(shape))
            out[off:off + n] = g[name].reshape(-1)
            off += n
    return out
