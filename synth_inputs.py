"""Seeded synthetic inputs for the stage-shard training step.

This module holds data recipes only: shard shapes, the parameter inventory of
one transformer layer, and counter-based random draws.  It contains none of
the layer mathematics and is imported by the tests, the benchmark and the CPU
checker alike so that every side starts from identical bits.

Shapes follow the paper's workloads (section 8.1 and Table 3: GPT models cut
by tensor and pipeline parallelism; a middle pipeline stage is a run of
identical transformer blocks, section 6.1).  One rank's share is described by
LOCAL sizes, i.e. after the tensor-parallel slice.

Draw recipe: every tensor has its own Philox stream keyed by
(seed, layer, tensor id); matrices ~ N(0, 0.02^2); norm gains 1 + N(0, 0.02^2);
biases and norm offsets N(0, 0.02^2) (non-zero so that their gradients are
exercised); stage input x ~ N(0, 1) laid out [seq, micro_batch, hidden];
output gradient dy ~ N(0, (1e-2)^2).  For bf16 presets each draw is snapped to
the bf16 grid by clearing the low 16 bits of its fp32 pattern, so both sides
start from values that bf16 storage represents exactly.
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, List, Tuple

import numpy as np

DTYPE_FP32 = 0
DTYPE_BF16 = 1
NORM_LAYERNORM = 0
NORM_RMSNORM = 1
ACT_GELU_TANH = 0
ACT_GELU_ERF = 1
ACT_SWIGLU = 2
POS_NONE = 0
POS_ROTARY = 1


@dataclasses.dataclass(frozen=True)
class StageConfig:
    """One rank's pipeline-stage shard; all sizes are local to the rank."""
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    seq: int
    micro_batch: int
    dtype: int = DTYPE_BF16
    norm: int = NORM_LAYERNORM
    act: int = ACT_GELU_TANH
    pos: int = POS_NONE
    has_bias: int = 1
    norm_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def tokens(self) -> int:
        return self.seq * self.micro_batch

    @property
    def attn_width(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def qkv_width(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def fc1_width(self) -> int:
        return 2 * self.ffn if self.act == ACT_SWIGLU else self.ffn

    def replace(self, **kw) -> "StageConfig":
        return dataclasses.replace(self, **kw)


PRESETS: Dict[str, StageConfig] = {
    # tiny GPT stage, fp32 end to end
    "tiny": StageConfig(2, 256, 4, 4, 64, 1024, 128, 2, dtype=DTYPE_FP32),
    # GPT 6.7B under TP=8: hidden 4096, 4 local heads, local FFN 2048
    "gpt6p7b": StageConfig(4, 4096, 4, 4, 128, 2048, 2048, 1),
    # GPT-3 175B under TP=8, 12 layers per pipeline stage
    "gpt175b": StageConfig(12, 12288, 12, 12, 128, 6144, 2048, 1),
    # Llama-70B under TP=8: GQA 8 q / 1 kv local heads, SwiGLU, RMSNorm, rotary
    "llama70b": StageConfig(10, 8192, 8, 1, 128, 3584, 4096, 1, norm=NORM_RMSNORM,
                            act=ACT_SWIGLU, pos=POS_ROTARY, has_bias=0),
    # long-context stress of the same shard
    "longctx": StageConfig(2, 8192, 8, 1, 128, 3584, 16384, 1, norm=NORM_RMSNORM,
                           act=ACT_SWIGLU, pos=POS_ROTARY, has_bias=0),
}

ADAM_DEFAULTS = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0)
ADAM_SWEEP_ELEMS = 1_200_000_000
BASE_SEED = 1234


def layer_inventory(cfg: StageConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of one layer's parameter tensors, in flat-buffer order."""
    h, A, Nqkv, F1, f = cfg.hidden, cfg.attn_width, cfg.qkv_width, cfg.fc1_width, cfg.ffn
    inv: List[Tuple[str, Tuple[int, ...]]] = [("norm1_gain", (h,))]
    if cfg.norm == NORM_LAYERNORM:
        inv.append(("norm1_offset", (h,)))
    inv.append(("w_qkv", (Nqkv, h)))
    if cfg.has_bias:
        inv.append(("b_qkv", (Nqkv,)))
    inv.append(("w_out", (h, A)))
    if cfg.has_bias:
        inv.append(("b_out", (h,)))
    inv.append(("norm2_gain", (h,)))
    if cfg.norm == NORM_LAYERNORM:
        inv.append(("norm2_offset", (h,)))
    inv.append(("w_fc1", (F1, h)))
    if cfg.has_bias:
        inv.append(("b_fc1", (F1,)))
    inv.append(("w_fc2", (h, f)))
    if cfg.has_bias:
        inv.append(("b_fc2", (h,)))
    return inv


def layer_param_count(cfg: StageConfig) -> int:
    return sum(int(np.prod(shape)) for _, shape in layer_inventory(cfg))


def stage_param_count(cfg: StageConfig) -> int:
    return cfg.n_layers * layer_param_count(cfg)


def _stream(seed: int, layer: int, tag: str) -> np.random.Generator:
    key = (int(seed) & 0xFFFFFFFF) | ((int(layer) & 0xFFFF) << 32) | ((zlib.crc32(tag.encode()) & 0xFFFF) << 48)
    return np.random.Generator(np.random.Philox(key=key))


def snap_to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Clear the low 16 bits of each fp32 pattern (values become bf16-exact)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 storage pattern of bf16-exact fp32 values (upper half of each word)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _finish(cfg: StageConfig, a: np.ndarray) -> np.ndarray:
    return snap_to_bf16_grid(a) if cfg.dtype == DTYPE_BF16 else a


def normal(seed: int, layer: int, tag: str, shape, std: float, mean: float = 0.0) -> np.ndarray:
    g = _stream(seed, layer, tag)
    a = g.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return a


def make_layer_params(cfg: StageConfig, layer: int, seed: int = BASE_SEED) -> Dict[str, np.ndarray]:
    """fp32 arrays (bf16-exact when cfg.dtype is bf16) for one layer, keyed by name."""
    out: Dict[str, np.ndarray] = {}
    for name, shape in layer_inventory(cfg):
        mean = 1.0 if name.endswith("_gain") else 0.0
        out[name] = _finish(cfg, normal(seed, layer, name, shape, 0.02, mean))
    return out


def make_flat_params(cfg: StageConfig, seed: int = BASE_SEED) -> np.ndarray:
    """All layers concatenated in inventory order (the library's flat layout)."""
    flat = np.empty(stage_param_count(cfg), dtype=np.float32)
    off = 0
    for layer in range(cfg.n_layers):
        p = make_layer_params(cfg, layer, seed)
        for name, shape in layer_inventory(cfg):
            n = int(np.prod(shape))
            flat[off:off + n] = p[name].reshape(-1)
            off += n
    return flat


def split_flat(cfg: StageConfig, flat: np.ndarray) -> List[Dict[str, np.ndarray]]:
    """Views of a flat buffer as per-layer dictionaries."""
    layers = []
    off = 0
    for _ in range(cfg.n_layers):
        d = {}
        for name, shape in layer_inventory(cfg):
            n = int(np.prod(shape))
            d[name] = flat[off:off + n].reshape(shape)
            off += n
        layers.append(d)
    return layers


def make_x(cfg: StageConfig, seed: int = BASE_SEED) -> np.ndarray:
    """Stage input, the tensor the previous pipeline stage would send: [seq, micro_batch, hidden]."""
    return _finish(cfg, normal(seed, 0xFFFF, "x", (cfg.seq, cfg.micro_batch, cfg.hidden), 1.0))


def make_dy(cfg: StageConfig, seed: int = BASE_SEED) -> np.ndarray:
    """Output gradient, the tensor the next pipeline stage would send back."""
    return _finish(cfg, normal(seed, 0xFFFF, "dy", (cfg.seq, cfg.micro_batch, cfg.hidden), 1e-2))


def make_adam_state(n: int, seed: int = BASE_SEED, chunk: int = 1 << 24):
    """Flat optimizer-sweep inputs: p ~ N(0, 0.02^2), g ~ N(0, (1e-3)^2), and
    non-zero moment buffers m ~ N(0, (1e-4)^2), v = 1e-3 z^2 with z ~ N(0, (1e-3)^2)
    (the magnitudes such buffers have early in training)."""
    p = np.empty(n, np.float32)
    g = np.empty(n, np.float32)
    m = np.empty(n, np.float32)
    v = np.empty(n, np.float32)
    for c, lo in enumerate(range(0, n, chunk)):
        hi = min(n, lo + chunk)
        p[lo:hi] = normal(seed, c, "adam_p", (hi - lo,), 0.02)
        g[lo:hi] = normal(seed, c, "adam_g", (hi - lo,), 1e-3)
        m[lo:hi] = normal(seed, c, "adam_m", (hi - lo,), 1e-4)
        z = normal(seed, c, "adam_z", (hi - lo,), 1e-3)
        v[lo:hi] = np.float32(1e-3) * z * z
    return p, g, m, v


# ---- mixture-of-experts MLP shard ------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class MoeConfig:
    """One rank's expert shard; sizes local to the rank except n_experts (global) and ep."""
    tokens: int
    hidden: int
    ffn: int
    n_experts: int
    ep: int
    top_k: int
    capacity: int
    dtype: int = DTYPE_BF16
    act: int = ACT_GELU_TANH
    has_bias: int = 1

    def replace(self, **kw) -> "MoeConfig":
        return dataclasses.replace(self, **kw)


def moe_capacity(tokens: int, top_k: int, n_experts: int, factor: float = 1.0) -> int:
    return max(1, -(-int(round(factor * tokens * top_k * 1000)) // (1000 * n_experts)))


# Shaped like the paper's largest workload (Table 3: 5.12T parameters, TP 8, PP 8, EP 16): 96 layers of 16 experts with
# 8 h^2 parameters each give 5.15e12 at hidden 20480; one rank holds one expert's tensor-parallel slice (4h / 8 = 10240
# columns) and sees one micro-batch of 2048 tokens; top-2 routing with capacity factor 1 (the paper states neither).
MOE_PRESETS = {
    "moe5t": MoeConfig(2048, 20480, 10240, 16, 16, 2, moe_capacity(2048, 2, 16)),
}


def moe_inventory(cfg: MoeConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    inv: List[Tuple[str, Tuple[int, ...]]] = [("w_router", (cfg.n_experts, cfg.hidden))]
    for j in range(cfg.n_experts // cfg.ep):
        inv.append((f"w_fc1.{j}", (cfg.ffn, cfg.hidden)))
        if cfg.has_bias:
            inv.append((f"b_fc1.{j}", (cfg.ffn,)))
        inv.append((f"w_fc2.{j}", (cfg.hidden, cfg.ffn)))
        if cfg.has_bias:
            inv.append((f"b_fc2.{j}", (cfg.hidden,)))
    return inv


def make_moe_params(cfg: MoeConfig, seed: int = BASE_SEED, router_std: float = 0.02) -> Dict[str, np.ndarray]:
    """N(0, 0.02^2) everywhere (the router too unless told otherwise), snapped to the bf16 grid for bf16 shards."""
    out: Dict[str, np.ndarray] = {}
    for name, shape in moe_inventory(cfg):
        a = normal(seed, 0x4D6F, name, shape, router_std if name == "w_router" else 0.02)
        out[name] = snap_to_bf16_grid(a) if cfg.dtype == DTYPE_BF16 else a
    return out


def make_moe_io(cfg: MoeConfig, seed: int = BASE_SEED):
    """Layer input c ~ N(0, 1) (a normalised residual stream) and output gradient ~ N(0, 1e-4), [tokens, hidden]."""
    fin = (lambda a: snap_to_bf16_grid(a)) if cfg.dtype == DTYPE_BF16 else (lambda a: a)
    return (fin(normal(seed, 0x4D6F, "moe_c", (cfg.tokens, cfg.hidden), 1.0)),
            fin(normal(seed, 0x4D6F, "moe_dout", (cfg.tokens, cfg.hidden), 1e-2)))
