"""fp64 CPU checker for one pipeline-stage shard's training iteration.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
GPU library is compared against; nothing on the product path may import it.

What it defines.  The paper (section 4.2) runs "a full shadow iteration" of a
rank's model partition inside a communication-free sandbox: forward, backward
and optimizer step, with every tensor that would cross the sandbox boundary
supplied from outside and `send`/`barrier` skipped.  For a middle pipeline
stage the partition is a run of identical transformer blocks (section 6.1) and
the state is parameters plus optimizer states (section 7, State
Synchronization).  The paper does not spell out the layer mathematics; it is
the Megatron-style pre-norm GPT block (and its Llama variant) written out
below from the textbook definitions:

    a   = Norm(x; gain1, offset1)
    qkv = a Wqkv^T + bqkv            columns [Q | K | V], heads contiguous
    q,k = Rotary(q), Rotary(k)       (Llama variant only)
    ctx = causal softmax(q k^T / sqrt(d)) v   per (batch entry, head); GQA shares kv heads
    x1  = x + ctx Wout^T + bout      (the tensor-parallel all-reduce is the identity)
    c   = Norm(x1; gain2, offset2)
    g   = gelu(c W1^T + b1)          or  silu(c Wgate^T) * (c Wup^T)
    y   = x1 + g W2^T + b2           (all-reduce = identity again)

followed, after the hand-derived backward pass, by Adam with bias correction
on fp32 master weights and a round-to-nearest-even bf16 copy.

Everything is numpy float64.  Matrix products go to the host BLAS through `@`;
nothing is blocked, fused or reordered.  Attention is evaluated one (batch
entry, head) at a time on the full s x s score matrix.

Pins (tests/test_oracle_pins.py): central finite differences for every
gradient, an independent pure-loop evaluation on tiny shapes, softmax row sums
and causal zeros, closed-form attention cases, tensor-parallel re-assembly
into the unsharded layer, closed-form Adam steps, hand-picked bf16 rounding
patterns; for the multi-micro-batch iteration: additivity of the gradients,
hand-computed clipping factors, the slices tiling the state exactly once.
End-to-end values at the large presets have no external pin beyond those (the
paper prints no numbers for this path).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Tuple

import numpy as np
from scipy.special import erf as _scipy_erf

F64 = np.float64

# enumerations mirror the public C header's integer codes
NORM_LAYERNORM, NORM_RMSNORM = 0, 1
ACT_GELU_TANH, ACT_GELU_ERF, ACT_SWIGLU = 0, 1, 2
POS_NONE, POS_ROTARY = 0, 1


# ----------------------------------------------------------------------------
# normalisation
# ----------------------------------------------------------------------------
def norm_fwd(x: np.ndarray, gain: np.ndarray, offset: Optional[np.ndarray], kind: int, eps: float):
    """LayerNorm (biased variance) or RMSNorm over the last axis.

    Returns (out, xhat, rstd).  xhat is the normalised input before the affine map."""
    x = np.asarray(x, F64)
    if kind == NORM_LAYERNORM:
        mu = x.mean(axis=-1, keepdims=True)
        var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
        rstd = 1.0 / np.sqrt(var + eps)
        xhat = (x - mu) * rstd
        out = xhat * gain + offset
    else:
        ms = (x * x).mean(axis=-1, keepdims=True)
        rstd = 1.0 / np.sqrt(ms + eps)
        xhat = x * rstd
        out = xhat * gain
    return out, xhat, rstd


def norm_bwd(dout: np.ndarray, xhat: np.ndarray, rstd: np.ndarray, gain: np.ndarray, kind: int):
    """Gradient of norm_fwd.  Returns (dx, dgain, doffset or None)."""
    dout = np.asarray(dout, F64)
    w = dout * gain
    dgain = (dout * xhat).reshape(-1, xhat.shape[-1]).sum(axis=0)
    if kind == NORM_LAYERNORM:
        doffset = dout.reshape(-1, dout.shape[-1]).sum(axis=0)
        dx = (w - w.mean(axis=-1, keepdims=True) - xhat * (w * xhat).mean(axis=-1, keepdims=True)) * rstd
    else:
        doffset = None
        dx = (w - xhat * (w * xhat).mean(axis=-1, keepdims=True)) * rstd
    return dx, dgain, doffset


# ----------------------------------------------------------------------------
# activations
# ----------------------------------------------------------------------------
_K_GELU = math.sqrt(2.0 / math.pi)


def _erf(u: np.ndarray) -> np.ndarray:
    return _scipy_erf(u)


def gelu_fwd(u: np.ndarray, kind: int) -> np.ndarray:
    if kind == ACT_GELU_TANH:
        return 0.5 * u * (1.0 + np.tanh(_K_GELU * (u + 0.044715 * u ** 3)))
    return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))


def gelu_bwd(dg: np.ndarray, u: np.ndarray, kind: int) -> np.ndarray:
    if kind == ACT_GELU_TANH:
        th = np.tanh(_K_GELU * (u + 0.044715 * u ** 3))
        return dg * (0.5 * (1.0 + th) + 0.5 * u * (1.0 - th * th) * _K_GELU * (1.0 + 3 * 0.044715 * u * u))
    pdf = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    return dg * (0.5 * (1.0 + _erf(u / math.sqrt(2.0))) + u * pdf)


def _sigmoid(z: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-z))


def swiglu_fwd(u_gate: np.ndarray, u_up: np.ndarray) -> np.ndarray:
    return u_gate * _sigmoid(u_gate) * u_up


def swiglu_bwd(dg: np.ndarray, u_gate: np.ndarray, u_up: np.ndarray):
    sg = _sigmoid(u_gate)
    du_up = dg * u_gate * sg
    du_gate = dg * u_up * sg * (1.0 + u_gate * (1.0 - sg))
    return du_gate, du_up


# ----------------------------------------------------------------------------
# rotary positions (rotate-half pairing: element j with element j + d/2)
# ----------------------------------------------------------------------------
def rotary_angles(seq: int, head_dim: int, theta: float) -> np.ndarray:
    j = np.arange(head_dim // 2, dtype=F64)
    inv_freq = theta ** (-2.0 * j / head_dim)
    return np.arange(seq, dtype=F64)[:, None] * inv_freq[None, :]     # [seq, d/2]


def rotary_apply(z: np.ndarray, angles: np.ndarray, sign: float = 1.0) -> np.ndarray:
    """z: [seq, ..., d]; rotates pair (j, j+d/2) at position i by sign*angles[i, j]."""
    d = z.shape[-1]
    shape = (z.shape[0],) + (1,) * (z.ndim - 2) + (d // 2,)
    cos = np.cos(angles).reshape(shape)
    sin = sign * np.sin(angles).reshape(shape)
    lo, hi = z[..., : d // 2], z[..., d // 2:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


# ----------------------------------------------------------------------------
# causal attention on one (batch entry, head)
# ----------------------------------------------------------------------------
def causal_probs(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Row softmax of q k^T / sqrt(d) with entries j > i removed.  q, k: [s, d]."""
    s, d = q.shape
    scores = (q @ k.T) / math.sqrt(d)
    scores = np.where(np.tril(np.ones((s, s), dtype=bool)), scores, -np.inf)
    scores = scores - scores.max(axis=1, keepdims=True)
    e = np.exp(scores)
    return e / e.sum(axis=1, keepdims=True)


def attention_fwd(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """q: [s, b, nq, d]; k, v: [s, b, nkv, d] -> ctx [s, b, nq, d]."""
    s, b, nq, d = q.shape
    group = nq // k.shape[2]
    ctx = np.empty_like(q)
    for n in range(b):
        for g in range(nq):
            kap = g // group
            p = causal_probs(q[:, n, g], k[:, n, kap])
            ctx[:, n, g] = p @ v[:, n, kap]
    return ctx


def attention_bwd(dctx: np.ndarray, q: np.ndarray, k: np.ndarray, v: np.ndarray):
    """Gradients (dq, dk, dv) of attention_fwd; probabilities are re-evaluated."""
    s, b, nq, d = q.shape
    group = nq // k.shape[2]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    inv = 1.0 / math.sqrt(d)
    for n in range(b):
        for g in range(nq):
            kap = g // group
            p = causal_probs(q[:, n, g], k[:, n, kap])
            dc = dctx[:, n, g]
            dv[:, n, kap] += p.T @ dc
            dp = dc @ v[:, n, kap].T
            dsc = p * (dp - (dp * p).sum(axis=1, keepdims=True))
            dq[:, n, g] = dsc @ k[:, n, kap] * inv
            dk[:, n, kap] += dsc.T @ q[:, n, g] * inv
    return dq, dk, dv


# ----------------------------------------------------------------------------
# one transformer layer
# ----------------------------------------------------------------------------
def _get(p: Dict[str, np.ndarray], name: str):
    a = p.get(name)
    return None if a is None else np.asarray(a, F64)


def layer_fwd(cfg, p: Dict[str, np.ndarray], x: np.ndarray):
    """x: [s, b, h] -> (y, stash).  cfg needs the attribute names of the public
    stage configuration (hidden, n_q_heads, n_kv_heads, head_dim, ffn, norm, act, pos,
    has_bias, norm_eps, rope_theta)."""
    x = np.asarray(x, F64)
    s, b, h = x.shape
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    A = nq * d
    st: Dict[str, np.ndarray] = {"x": x}

    a, st["xhat1"], st["rstd1"] = norm_fwd(x, _get(p, "norm1_gain"), _get(p, "norm1_offset"), cfg.norm, cfg.norm_eps)
    st["a"] = a
    qkv = a @ _get(p, "w_qkv").T
    if cfg.has_bias:
        qkv = qkv + _get(p, "b_qkv")
    q = qkv[..., :A].reshape(s, b, nq, d)
    k = qkv[..., A:A + nkv * d].reshape(s, b, nkv, d)
    v = qkv[..., A + nkv * d:].reshape(s, b, nkv, d)
    if cfg.pos == POS_ROTARY:
        ang = rotary_angles(s, d, cfg.rope_theta)
        q, k = rotary_apply(q, ang), rotary_apply(k, ang)
    st["q"], st["k"], st["v"] = q, k, v
    ctx = attention_fwd(q, k, v).reshape(s, b, A)
    st["ctx"] = ctx
    x1 = x + ctx @ _get(p, "w_out").T
    if cfg.has_bias:
        x1 = x1 + _get(p, "b_out")
    st["x1"] = x1

    c, st["xhat2"], st["rstd2"] = norm_fwd(x1, _get(p, "norm2_gain"), _get(p, "norm2_offset"), cfg.norm, cfg.norm_eps)
    st["c"] = c
    u = c @ _get(p, "w_fc1").T
    if cfg.has_bias:
        u = u + _get(p, "b_fc1")
    st["u"] = u
    if cfg.act == ACT_SWIGLU:
        g = swiglu_fwd(u[..., :cfg.ffn], u[..., cfg.ffn:])
    else:
        g = gelu_fwd(u, cfg.act)
    st["g"] = g
    y = x1 + g @ _get(p, "w_fc2").T
    if cfg.has_bias:
        y = y + _get(p, "b_fc2")
    return y, st


def layer_bwd(cfg, p: Dict[str, np.ndarray], st: Dict[str, np.ndarray], dy: np.ndarray):
    """Returns (dx, grads) where grads maps every parameter name to its gradient."""
    dy = np.asarray(dy, F64)
    s, b, h = dy.shape
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    A = nq * d
    T = s * b
    gr: Dict[str, np.ndarray] = {}
    flat = lambda t: t.reshape(T, -1)

    # y = x1 + g W2^T + b2
    dg = dy @ _get(p, "w_fc2")
    gr["w_fc2"] = flat(dy).T @ flat(st["g"])
    if cfg.has_bias:
        gr["b_fc2"] = flat(dy).sum(axis=0)
    dx1 = dy.copy()

    # activation and first MLP matrix
    u = st["u"]
    if cfg.act == ACT_SWIGLU:
        du_gate, du_up = swiglu_bwd(dg, u[..., :cfg.ffn], u[..., cfg.ffn:])
        du = np.concatenate([du_gate, du_up], axis=-1)
    else:
        du = gelu_bwd(dg, u, cfg.act)
    dc = du @ _get(p, "w_fc1")
    gr["w_fc1"] = flat(du).T @ flat(st["c"])
    if cfg.has_bias:
        gr["b_fc1"] = flat(du).sum(axis=0)

    # second norm
    dn, gr["norm2_gain"], doff = norm_bwd(dc, st["xhat2"], st["rstd2"], _get(p, "norm2_gain"), cfg.norm)
    if doff is not None:
        gr["norm2_offset"] = doff
    dx1 = dx1 + dn

    # x1 = x + ctx Wout^T + bout
    dctx = dx1 @ _get(p, "w_out")
    gr["w_out"] = flat(dx1).T @ flat(st["ctx"])
    if cfg.has_bias:
        gr["b_out"] = flat(dx1).sum(axis=0)

    # attention and rotary
    dq, dk, dv = attention_bwd(dctx.reshape(s, b, nq, d), st["q"], st["k"], st["v"])
    if cfg.pos == POS_ROTARY:
        ang = rotary_angles(s, d, cfg.rope_theta)
        dq, dk = rotary_apply(dq, ang, -1.0), rotary_apply(dk, ang, -1.0)
    dqkv = np.concatenate([dq.reshape(s, b, A), dk.reshape(s, b, nkv * d), dv.reshape(s, b, nkv * d)], axis=-1)

    # qkv projection
    da = dqkv @ _get(p, "w_qkv")
    gr["w_qkv"] = flat(dqkv).T @ flat(st["a"])
    if cfg.has_bias:
        gr["b_qkv"] = flat(dqkv).sum(axis=0)

    # first norm
    dn, gr["norm1_gain"], doff = norm_bwd(da, st["xhat1"], st["rstd1"], _get(p, "norm1_gain"), cfg.norm)
    if doff is not None:
        gr["norm1_offset"] = doff
    dx = dx1 + dn
    return dx, gr


# ----------------------------------------------------------------------------
# the stage: layers in sequence, no final norm (middle pipeline stage)
# ----------------------------------------------------------------------------
def stage_fwd(cfg, layers: List[Dict[str, np.ndarray]], x: np.ndarray):
    stashes = []
    for p in layers:
        x, st = layer_fwd(cfg, p, x)
        stashes.append(st)
    return x, stashes


def stage_bwd(cfg, layers: List[Dict[str, np.ndarray]], stashes, dy: np.ndarray):
    grads = [None] * len(layers)
    for i in reversed(range(len(layers))):
        dy, grads[i] = layer_bwd(cfg, layers[i], stashes[i], dy)
    return dy, grads


# ----------------------------------------------------------------------------
# Adam on fp32 master weights, with a bf16 copy for the next forward pass
# ----------------------------------------------------------------------------
def adam_step(p, g, m, v, step: int, lr: float, beta1: float, beta2: float, eps: float,
              weight_decay: float = 0.0, grad_scale: float = 1.0):
    """One bias-corrected Adam update (decoupled weight decay), all in fp64.
    Returns new (p, m, v)."""
    p, g, m, v = (np.asarray(t, F64) for t in (p, g, m, v))
    gs = grad_scale * g
    m = beta1 * m + (1.0 - beta1) * gs
    v = beta2 * v + (1.0 - beta2) * gs * gs
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    p = p - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * p)
    return p, m, v


# ----------------------------------------------------------------------------
# A whole iteration as the paper's default profiles run it (section 8.1): several
# micro-batches whose gradients add up, gradient-norm clipping, and the optimizer
# step on this data-parallel rank's share of the state (distributed optimizer)
# ----------------------------------------------------------------------------
def grad_sq_sum(flat_grads: np.ndarray) -> float:
    """Sum of squares of a gradient vector (this rank's contribution to the squared global norm; the
    sum over ranks that would follow is served locally, i.e. it is the identity here)."""
    g = np.asarray(flat_grads, F64)
    return float(np.dot(g, g))


def clip_scale(sq_sum: float, max_norm: float, eps: float = 1e-6) -> float:
    """Factor that brings a gradient of squared norm sq_sum down to norm max_norm: min(1, c / (|g| + eps)).
    (Clipping by global norm; the paper does not restate the rule, this is the usual one with the small
    constant in the denominator.)  max_norm <= 0 switches clipping off."""
    if max_norm <= 0.0:
        return 1.0
    return min(1.0, max_norm / (float(np.sqrt(sq_sum)) + eps))


def optimizer_slice(n: int, dp: int, rank: int):
    """[first, first+count) of the flat state that data-parallel rank `rank` of `dp` updates: equal
    contiguous shares of ceil(n / dp) rounded up to 8 elements, the last one short."""
    share = -(-n // dp)
    share = -(-share // 8) * 8
    first = min(n, rank * share)
    return first, min(n, first + share) - first


def accumulate_micro_batches(cfg, layers, xs, dys):
    """Forward and backward over every micro-batch (xs[i], dys[i]); the parameter gradients add up.
    Returns (list of y, list of dx, per-layer gradient dicts)."""
    ys, dxs, total = [], [], None
    for x, dy in zip(xs, dys):
        y, stashes = stage_fwd(cfg, layers, x)
        dx, grads = stage_bwd(cfg, layers, stashes, dy)
        ys.append(y)
        dxs.append(dx)
        if total is None:
            total = grads
        else:
            total = [{k: total[l][k] + grads[l][k] for k in grads[l]} for l in range(len(grads))]
    return ys, dxs, total


def iteration_update(p, g, m, v, step: int, hp: Dict[str, float], max_norm: float, n_micro: int, dp: int, rank: int):
    """Optimizer part of the iteration on flat fp64 vectors: the accumulated gradient g is averaged over
    the n_micro micro-batches and clipped by its global norm (both as ONE factor handed to Adam), and only
    this rank's slice of p, m, v changes.  Returns (p, m, v, factor, first, count)."""
    p, g, m, v = (np.array(t, F64) for t in (p, g, m, v))
    avg = 1.0 / n_micro
    factor = avg * clip_scale(grad_sq_sum(g) * avg * avg, max_norm)
    first, count = optimizer_slice(p.size, dp, rank)
    sl = slice(first, first + count)
    p[sl], m[sl], v[sl] = adam_step(p[sl], g[sl], m[sl], v[sl], step, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                                    hp.get("weight_decay", 0.0), factor)
    return p, m, v, factor, first, count


def bf16_round_nearest_even(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (ties to even); returns the uint16 patterns.
    Finite inputs only."""
    bits = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    return rounded.astype(np.uint16)


def bf16_to_f64(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(F64)
