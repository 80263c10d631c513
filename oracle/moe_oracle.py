"""fp64 CPU checker for one rank's mixture-of-experts MLP shard.

TEST INFRASTRUCTURE ONLY: the slow, plain definition the GPU library is compared against; nothing on
the product path may import it.

What it defines.  The paper's largest workloads (Table 3: 960B to 5.12T parameters, expert parallelism
2 to 16) are mixture-of-experts GPT models; section 4.2 notes that token routing depends on the input
but that the frameworks pre-allocate FIXED-SIZE expert buffers, so memory layout and communication
structure stay static and the sandbox warm-up covers them.  The paper gives no layer mathematics; this
is the Megatron-style token-choice layer with capacity, in the form one rank runs inside the sandbox
(every collective served locally, section 4.2), replacing the dense MLP of stage_oracle.py:

  router     logits[t, e] = c[t] . Wr[e]                 E global experts
             choose the k largest logits of a token (ties: the lower expert index first)
             gate[t, i]   = softmax over the k chosen logits
  dispatch   expert e owns a buffer of C rows.  Assignments are taken in token order (and, within a
             token, in order of decreasing logit); an assignment gets the next free row of its expert's
             buffer, or is DROPPED when the buffer is full.  Unused rows are zero.
  exchange   the all-to-all that would carry buffer e to the rank holding expert e is the identity: the
             rank processes all E buffers itself, buffer e with its local expert e mod E_local
             (E_local = E / EP experts per rank; global expert e is local expert e mod E_local of rank
             e div E_local)
  expert     o = gelu(buf W1^T + b1) W2^T + b2            per buffer, with that local expert's weights
  combine    out[t] = sum over the token's kept assignments of gate * o[row of the assignment]

Backward pass derived by hand below; the routing decision is piecewise constant and gets no gradient,
the gates do (through the softmax over the chosen logits).  Everything is numpy float64; products go to
the host BLAS through `@`; nothing is blocked or fused.

Pins (tests/test_oracle_pins.py): central finite differences for every gradient; one expert with k = 1
equals the dense MLP of stage_oracle; k = E with room for everything equals the dense softmax mixture
written out directly; a crafted router that sends every token to one expert keeps exactly the first C;
expert-parallel groups equal the same layer with the shared weights written out per global expert.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np

from oracle import stage_oracle as so

F64 = np.float64


def router(c: np.ndarray, w_router: np.ndarray, k: int):
    """c [T, h], w_router [E, h] -> logits [T, E], idx [T, k] (decreasing logit, ties to the lower index),
    gates [T, k] = softmax over the chosen logits."""
    logits = np.asarray(c, F64) @ np.asarray(w_router, F64).T
    idx = np.argsort(-logits, axis=1, kind="stable")[:, :k]
    chosen = np.take_along_axis(logits, idx, axis=1)
    ex = np.exp(chosen - chosen.max(axis=1, keepdims=True))
    return logits, idx, ex / ex.sum(axis=1, keepdims=True)


def dispatch_plan(idx: np.ndarray, n_experts: int, capacity: int) -> np.ndarray:
    """row[t, i] = e * capacity + position inside expert e's buffer, or -1 when the assignment is dropped."""
    T, k = idx.shape
    used = [0] * n_experts
    row = np.full((T, k), -1, dtype=np.int64)
    for t in range(T):
        for i in range(k):
            e = int(idx[t, i])
            if used[e] < capacity:
                row[t, i] = e * capacity + used[e]
                used[e] += 1
    return row


def moe_fwd(c: np.ndarray, p: Dict[str, np.ndarray], n_experts: int, ep: int, k: int, capacity: int, act: int):
    """c [T, h].  p: 'w_router' [E, h]; per local expert j 'w_fc1.j' [f, h], 'b_fc1.j' [f], 'w_fc2.j' [h, f],
    'b_fc2.j' [h] (biases optional).  Returns (out [T, h], stash)."""
    c = np.asarray(c, F64)
    T, h = c.shape
    e_local = n_experts // ep
    logits, idx, gates = router(c, p["w_router"], k)
    row = dispatch_plan(idx, n_experts, capacity)
    buf = np.zeros((n_experts * capacity, h))
    for t in range(T):
        for i in range(k):
            if row[t, i] >= 0:
                buf[row[t, i]] = c[t]
    u, g, o = [None] * n_experts, [None] * n_experts, np.zeros((n_experts * capacity, h))
    for e in range(n_experts):
        j = e % e_local
        rows = slice(e * capacity, (e + 1) * capacity)
        u[e] = buf[rows] @ np.asarray(p[f"w_fc1.{j}"], F64).T
        if f"b_fc1.{j}" in p:
            u[e] = u[e] + np.asarray(p[f"b_fc1.{j}"], F64)
        g[e] = so.gelu_fwd(u[e], act)
        o[rows] = g[e] @ np.asarray(p[f"w_fc2.{j}"], F64).T
        if f"b_fc2.{j}" in p:
            o[rows] = o[rows] + np.asarray(p[f"b_fc2.{j}"], F64)
    out = np.zeros((T, h))
    for t in range(T):
        for i in range(k):
            if row[t, i] >= 0:
                out[t] += gates[t, i] * o[row[t, i]]
    st = {"c": c, "logits": logits, "idx": idx, "gates": gates, "row": row, "buf": buf, "u": u, "g": g, "o": o}
    return out, st


def moe_bwd(dout: np.ndarray, p: Dict[str, np.ndarray], st, n_experts: int, ep: int, k: int, capacity: int, act: int):
    """Returns (dc [T, h], grads keyed like p)."""
    dout = np.asarray(dout, F64)
    c, idx, gates, row = st["c"], st["idx"], st["gates"], st["row"]
    T, h = c.shape
    e_local = n_experts // ep
    gr = {name: np.zeros(np.shape(a)) for name, a in p.items()}
    # combine
    d_o = np.zeros((n_experts * capacity, h))
    dgate = np.zeros((T, k))
    for t in range(T):
        for i in range(k):
            if row[t, i] >= 0:
                d_o[row[t, i]] = gates[t, i] * dout[t]
                dgate[t, i] = dout[t] @ st["o"][row[t, i]]
    # experts
    dbuf = np.zeros((n_experts * capacity, h))
    for e in range(n_experts):
        j = e % e_local
        rows = slice(e * capacity, (e + 1) * capacity)
        dg = d_o[rows] @ np.asarray(p[f"w_fc2.{j}"], F64)
        gr[f"w_fc2.{j}"] += d_o[rows].T @ st["g"][e]
        if f"b_fc2.{j}" in p:
            gr[f"b_fc2.{j}"] += d_o[rows].sum(axis=0)
        du = so.gelu_bwd(dg, st["u"][e], act)
        dbuf[rows] = du @ np.asarray(p[f"w_fc1.{j}"], F64)
        gr[f"w_fc1.{j}"] += du.T @ st["buf"][rows]
        if f"b_fc1.{j}" in p:
            gr[f"b_fc1.{j}"] += du.sum(axis=0)
    # dispatch
    dc = np.zeros((T, h))
    for t in range(T):
        for i in range(k):
            if row[t, i] >= 0:
                dc[t] += dbuf[row[t, i]]
    # router: softmax over the chosen logits
    dchosen = gates * (dgate - (gates * dgate).sum(axis=1, keepdims=True))
    dlogits = np.zeros_like(st["logits"])
    np.put_along_axis(dlogits, idx, dchosen, axis=1)
    gr["w_router"] += dlogits.T @ c
    dc += dlogits @ np.asarray(p["w_router"], F64)
    return dc, gr


def min_decision_margin(logits: np.ndarray, k: int) -> float:
    """Smallest gap between adjacent logits among a token's k + 1 largest: how far the inputs are from a different
    choice or a different order of the chosen experts (used by tests to state their precondition)."""
    top = -np.sort(-np.asarray(logits, F64), axis=1)[:, :k + 1]
    return float((top[:, :-1] - top[:, 1:]).min())
