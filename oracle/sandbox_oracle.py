"""fp64 CPU checker for the record / replay layer of the communication-free sandbox.

TEST INFRASTRUCTURE ONLY: the slow, plain definition the GPU library is compared against; nothing on
the product path may import it.

What it defines.  The paper (section 4.2) places a hook between the training framework and the
collective library.  In the pre-record step the hook stores the OUTPUT tensor of every collective
call once it has completed.  In the replay step a joiner runs a shadow iteration alone: a call that
would reach outside the sandbox is answered with the stored tensor, `send` and `barrier` are skipped
because they do not change the caller's state.  Section 4.3 narrows the scope: only communication
edges that cross the sandbox boundary are recorded / loaded (intra-machine tensor-parallel traffic
runs natively; a batch of machines that migrates together keeps its internal traffic real).

The shadow iteration written out here is stage_oracle's layer with its collective call sites made
explicit (Megatron-style tensor parallelism without sequence parallelism; numbering in call order):

  forward   recv(x)                       pipeline scope, what the previous stage sends
            per layer   part = ctx Wout^T -> all_reduce(part)   tensor scope;   x1 = x + part + bout
                        part = g W2^T     -> all_reduce(part)   tensor scope;   y  = x1 + part + b2
            send(y)                       pipeline scope
  backward  recv(dy)                      pipeline scope
            per layer   dc = du W1        -> all_reduce(dc)     tensor scope (input of a column-parallel map)
                        da = dqkv Wqkv    -> all_reduce(da)     tensor scope
            send(dx)                      pipeline scope
  update    all_reduce(flat gradient)     data scope;  barrier

A row-parallel map's bias is added after the all-reduce (once, not per rank).  A collective object
decides what each call returns:
  PassThrough   every call returns its local input (the degenerate sandbox of stage_oracle.py)
  Recorder      wraps another collective object; stores what it returned for the scopes it records
  Replayer      scopes on the boundary: the stored tensor, in call order, after checking that the call
                matches the stored one (kind, scope, site, shape); other scopes: the wrapped object
  ThreadGroup   a REAL group of ranks in one process (threads + barriers), used by the pins only

Pins (tests/test_oracle_pins.py): with PassThrough the hooked layer equals stage_oracle's layer
exactly; two tensor-parallel ranks run as a real group, rank 0 recording, and rank 0 replaying alone
reproduces its outputs, input gradient and parameter gradients of the real run bit for bit (the
paper's claim that replay yields valid state); a replay whose call sequence differs raises.
"""
from __future__ import annotations

import threading
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from oracle import stage_oracle as so

F64 = np.float64

# integer codes mirror the public C header
SCOPE_TP, SCOPE_PP, SCOPE_DP = 1, 2, 4
ALL_REDUCE, RECV, SEND, BARRIER = 0, 1, 2, 3
# call sites
SITE_X, SITE_Y, SITE_DY, SITE_DX, SITE_ATTN_OUT, SITE_MLP_OUT, SITE_D_MLP_IN, SITE_D_ATTN_IN, SITE_GRADS, SITE_STEP_END = range(10)


class PassThrough:
    """No peers: an all-reduce or a receive returns the caller's own tensor."""

    def call(self, kind: int, scope: int, site: int, t: Optional[np.ndarray]) -> Optional[np.ndarray]:
        return t


class ThreadGroup:
    """A real tensor-parallel group inside one process: each rank runs in its own thread; all_reduce adds the
    ranks' tensors in rank order.  Pipeline / data scope calls fall through to `outer`."""

    def __init__(self, n_ranks: int):
        self.n = n_ranks
        self.slots: List[Optional[np.ndarray]] = [None] * n_ranks
        self.barrier = threading.Barrier(n_ranks)

    def member(self, rank: int, outer=None):
        group = self

        class Member:
            def call(self, kind, scope, site, t):
                if scope != SCOPE_TP or kind != ALL_REDUCE:
                    return (outer or PassThrough()).call(kind, scope, site, t)
                group.slots[rank] = t
                group.barrier.wait()
                total = np.zeros_like(t)
                for r in range(group.n):
                    total = total + group.slots[r]
                group.barrier.wait()
                return total

        return Member()


class Recorder:
    """Pre-record step: stores the result of every receive / all-reduce whose scope is in `scopes`."""

    def __init__(self, inner, scopes: int):
        self.inner, self.scopes = inner, scopes
        self.tape: List[Tuple[int, int, int, np.ndarray]] = []

    def call(self, kind, scope, site, t):
        out = self.inner.call(kind, scope, site, t)
        if kind in (ALL_REDUCE, RECV) and (scope & self.scopes):
            self.tape.append((kind, scope, site, np.array(out, F64, copy=True)))
        return out


class ReplayMismatch(RuntimeError):
    pass


class Replayer:
    """Replay step: scopes in `boundary` are answered from the tape (entries of other scopes are never loaded),
    send and barrier on the boundary are skipped, everything else runs on `inner`."""

    def __init__(self, tape: Sequence[Tuple[int, int, int, np.ndarray]], boundary: int, inner=None):
        self.entries = [e for e in tape if e[1] & boundary]
        self.boundary, self.inner, self.at = boundary, inner or PassThrough(), 0
        self.skipped = 0

    def call(self, kind, scope, site, t):
        if not (scope & self.boundary):
            return self.inner.call(kind, scope, site, t)
        if kind in (SEND, BARRIER):
            self.skipped += 1
            return t
        if self.at >= len(self.entries):
            raise ReplayMismatch("tape exhausted")
        k, sc, si_, data = self.entries[self.at]
        if (k, sc, si_) != (kind, scope, site) or data.shape != np.shape(t):
            raise ReplayMismatch(f"call {self.at}: tape holds {(k, sc, si_, data.shape)}, program asks {(kind, scope, site, np.shape(t))}")
        self.at += 1
        return data.copy()


# ----------------------------------------------------------------------------
# the layer with its collective call sites explicit
# ----------------------------------------------------------------------------
def layer_fwd(cfg, p: Dict[str, np.ndarray], x: np.ndarray, comm):
    x = np.asarray(x, F64)
    s, b, h = x.shape
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    A = nq * d
    get = lambda name: None if p.get(name) is None else np.asarray(p[name], F64)
    st: Dict[str, np.ndarray] = {"x": x}
    a, st["xhat1"], st["rstd1"] = so.norm_fwd(x, get("norm1_gain"), get("norm1_offset"), cfg.norm, cfg.norm_eps)
    st["a"] = a
    qkv = a @ get("w_qkv").T
    if cfg.has_bias:
        qkv = qkv + get("b_qkv")
    q = qkv[..., :A].reshape(s, b, nq, d)
    k = qkv[..., A:A + nkv * d].reshape(s, b, nkv, d)
    v = qkv[..., A + nkv * d:].reshape(s, b, nkv, d)
    if cfg.pos == so.POS_ROTARY:
        ang = so.rotary_angles(s, d, cfg.rope_theta)
        q, k = so.rotary_apply(q, ang), so.rotary_apply(k, ang)
    st["q"], st["k"], st["v"] = q, k, v
    ctx = so.attention_fwd(q, k, v).reshape(s, b, A)
    st["ctx"] = ctx
    part = comm.call(ALL_REDUCE, SCOPE_TP, SITE_ATTN_OUT, ctx @ get("w_out").T)
    x1 = x + part
    if cfg.has_bias:
        x1 = x1 + get("b_out")
    st["x1"] = x1
    c, st["xhat2"], st["rstd2"] = so.norm_fwd(x1, get("norm2_gain"), get("norm2_offset"), cfg.norm, cfg.norm_eps)
    st["c"] = c
    u = c @ get("w_fc1").T
    if cfg.has_bias:
        u = u + get("b_fc1")
    st["u"] = u
    g = so.swiglu_fwd(u[..., :cfg.ffn], u[..., cfg.ffn:]) if cfg.act == so.ACT_SWIGLU else so.gelu_fwd(u, cfg.act)
    st["g"] = g
    part = comm.call(ALL_REDUCE, SCOPE_TP, SITE_MLP_OUT, g @ get("w_fc2").T)
    y = x1 + part
    if cfg.has_bias:
        y = y + get("b_fc2")
    return y, st


def layer_bwd(cfg, p: Dict[str, np.ndarray], st: Dict[str, np.ndarray], dy: np.ndarray, comm):
    dy = np.asarray(dy, F64)
    s, b, h = dy.shape
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    A, T = nq * d, s * b
    get = lambda name: None if p.get(name) is None else np.asarray(p[name], F64)
    flat = lambda t: t.reshape(T, -1)
    gr: Dict[str, np.ndarray] = {}
    dg = dy @ get("w_fc2")
    gr["w_fc2"] = flat(dy).T @ flat(st["g"])
    if cfg.has_bias:
        gr["b_fc2"] = flat(dy).sum(axis=0)
    u = st["u"]
    if cfg.act == so.ACT_SWIGLU:
        du = np.concatenate(so.swiglu_bwd(dg, u[..., :cfg.ffn], u[..., cfg.ffn:]), axis=-1)
    else:
        du = so.gelu_bwd(dg, u, cfg.act)
    dc = comm.call(ALL_REDUCE, SCOPE_TP, SITE_D_MLP_IN, du @ get("w_fc1"))
    gr["w_fc1"] = flat(du).T @ flat(st["c"])
    if cfg.has_bias:
        gr["b_fc1"] = flat(du).sum(axis=0)
    dn, gr["norm2_gain"], doff = so.norm_bwd(dc, st["xhat2"], st["rstd2"], get("norm2_gain"), cfg.norm)
    if doff is not None:
        gr["norm2_offset"] = doff
    dx1 = dy + dn
    dctx = dx1 @ get("w_out")
    gr["w_out"] = flat(dx1).T @ flat(st["ctx"])
    if cfg.has_bias:
        gr["b_out"] = flat(dx1).sum(axis=0)
    dq, dk, dv = so.attention_bwd(dctx.reshape(s, b, nq, d), st["q"], st["k"], st["v"])
    if cfg.pos == so.POS_ROTARY:
        ang = so.rotary_angles(s, d, cfg.rope_theta)
        dq, dk = so.rotary_apply(dq, ang, -1.0), so.rotary_apply(dk, ang, -1.0)
    dqkv = np.concatenate([dq.reshape(s, b, A), dk.reshape(s, b, nkv * d), dv.reshape(s, b, nkv * d)], axis=-1)
    da = comm.call(ALL_REDUCE, SCOPE_TP, SITE_D_ATTN_IN, dqkv @ get("w_qkv"))
    gr["w_qkv"] = flat(dqkv).T @ flat(st["a"])
    if cfg.has_bias:
        gr["b_qkv"] = flat(dqkv).sum(axis=0)
    dn, gr["norm1_gain"], doff = so.norm_bwd(da, st["xhat1"], st["rstd1"], get("norm1_gain"), cfg.norm)
    if doff is not None:
        gr["norm1_offset"] = doff
    return dx1 + dn, gr


# ----------------------------------------------------------------------------
# the shadow iteration of one stage
# ----------------------------------------------------------------------------
def stage_fwd(cfg, layers, x_arg: np.ndarray, comm):
    x = comm.call(RECV, SCOPE_PP, SITE_X, np.asarray(x_arg, F64))
    stashes = []
    for p in layers:
        x, st = layer_fwd(cfg, p, x, comm)
        stashes.append(st)
    comm.call(SEND, SCOPE_PP, SITE_Y, x)
    return x, stashes


def stage_bwd(cfg, layers, stashes, dy_arg: np.ndarray, comm):
    dy = comm.call(RECV, SCOPE_PP, SITE_DY, np.asarray(dy_arg, F64))
    grads = [None] * len(layers)
    for i in reversed(range(len(layers))):
        dy, grads[i] = layer_bwd(cfg, layers[i], stashes[i], dy, comm)
    comm.call(SEND, SCOPE_PP, SITE_DX, dy)
    return dy, grads


def grad_sync(flat_grads: np.ndarray, comm) -> np.ndarray:
    """The data-parallel reduction of the flat gradient buffer, then the barrier that ends the step."""
    out = comm.call(ALL_REDUCE, SCOPE_DP, SITE_GRADS, np.asarray(flat_grads, F64))
    comm.call(BARRIER, SCOPE_DP, SITE_STEP_END, None)
    return out
