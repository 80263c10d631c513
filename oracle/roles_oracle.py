"""fp64 CPU checker for the layers that only the first and the last pipeline stage have.

TEST INFRASTRUCTURE ONLY: the slow, plain definition the GPU library is compared against; nothing on
the product path may import it.

What it defines.  With pipeline parallelism the paper (section 6.1) distinguishes three roles: the
middle stages are repeated transformer blocks (oracle/stage_oracle.py), the first stage additionally
holds the word-embedding layer and the last stage the output layer, the two sharing one shape (weight
tying).  The general standby warms all three roles (section 6.2).  The paper gives no mathematics for
these layers; they are written out here from the textbook definitions in the tensor-parallel form a
rank runs, with every collective served locally (section 4.2), i.e. replaced by the identity:

  first stage   x0[t] = W[token[t] - v0]          if v0 <= token[t] < v0 + V_local, else 0
                        (+ P[position(t)]         GPT presets: learned absolute positions)
                The all-reduce that would add the other ranks' rows is the identity.
  last stage    hn     = Norm(y; gain, offset)
                logits = hn W^T                    W [V_local, h], no bias
                loss_t = log sum_v exp(logits[t, v]) - (logits[t, target[t] - v0] if in range else 0)
                loss   = mean over tokens of loss_t
                The max / sum / target-logit all-reduces of the vocabulary-parallel cross-entropy are
                identities, so this is the cross-entropy over the rank's vocabulary shard.

Backward passes are derived by hand below.  Everything is numpy float64; products go to the host BLAS
through `@`; nothing is blocked or fused.

Pins (tests/test_oracle_pins.py): central finite differences for every gradient, the embedding
gradient against a dense one-hot product, closed forms of the cross-entropy (constant logits, one
dominant logit, targets outside the shard), row sums of the logit gradient.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from oracle import stage_oracle as so

F64 = np.float64


# ----------------------------------------------------------------------------
# first stage: vocabulary-parallel word embedding (+ learned positions)
# ----------------------------------------------------------------------------
def embedding_fwd(tokens: np.ndarray, w: np.ndarray, v0: int, pos_emb: Optional[np.ndarray]) -> np.ndarray:
    """tokens [s, b] integers; w [V_local, h] holds rows v0 .. v0+V_local-1 of the table; pos_emb
    [>= s, h] or None.  Returns x0 [s, b, h]."""
    tokens = np.asarray(tokens)
    w = np.asarray(w, F64)
    s, b = tokens.shape
    local = tokens - v0
    inside = (local >= 0) & (local < w.shape[0])
    x0 = np.where(inside[..., None], w[np.where(inside, local, 0)], 0.0)
    if pos_emb is not None:
        x0 = x0 + np.asarray(pos_emb, F64)[:s, None, :]
    return x0


def embedding_bwd(dx0: np.ndarray, tokens: np.ndarray, v_local: int, v0: int, n_pos: int):
    """Gradients of embedding_fwd: (dW [V_local, h], dP [n_pos, h] or None when n_pos == 0)."""
    dx0 = np.asarray(dx0, F64)
    tokens = np.asarray(tokens)
    s, b, h = dx0.shape
    dw = np.zeros((v_local, h), F64)
    for i in range(s):
        for n in range(b):
            r = int(tokens[i, n]) - v0
            if 0 <= r < v_local:
                dw[r] += dx0[i, n]
    dp = None
    if n_pos > 0:
        dp = np.zeros((n_pos, h), F64)
        dp[:s] = dx0.sum(axis=1)
    return dw, dp


# ----------------------------------------------------------------------------
# last stage: final norm, output layer, vocabulary-parallel cross-entropy
# ----------------------------------------------------------------------------
def xent_fwd(logits: np.ndarray, targets: np.ndarray, v0: int):
    """logits [T, V_local], targets [T] integers (global vocabulary ids).  Returns (loss_t [T], probs)."""
    logits = np.asarray(logits, F64)
    targets = np.asarray(targets).reshape(-1)
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    z = e.sum(axis=1, keepdims=True)
    lse = (m + np.log(z)).reshape(-1)
    local = targets - v0
    inside = (local >= 0) & (local < logits.shape[1])
    picked = np.where(inside, logits[np.arange(logits.shape[0]), np.where(inside, local, 0)], 0.0)
    return lse - picked, e / z


def xent_bwd(probs: np.ndarray, targets: np.ndarray, v0: int, dloss_t: np.ndarray) -> np.ndarray:
    """d loss_t / d logits, times dloss_t [T]: probs - onehot(target) where the target is in the shard."""
    targets = np.asarray(targets).reshape(-1)
    d = np.array(probs, F64)
    local = targets - v0
    inside = (local >= 0) & (local < d.shape[1])
    rows = np.arange(d.shape[0])[inside]
    d[rows, local[inside]] -= 1.0
    return d * np.asarray(dloss_t, F64).reshape(-1, 1)


def head_fwd(kind: int, eps: float, y: np.ndarray, gain: np.ndarray, offset: Optional[np.ndarray], w: np.ndarray,
             targets: np.ndarray, v0: int):
    """y [s, b, h] -> (loss, stash).  targets [s, b]."""
    s, b, h = y.shape
    hn, xhat, rstd = so.norm_fwd(y, gain, offset, kind, eps)
    logits = hn.reshape(s * b, h) @ np.asarray(w, F64).T
    loss_t, probs = xent_fwd(logits, np.asarray(targets).reshape(-1), v0)
    stash = dict(hn=hn, xhat=xhat, rstd=rstd, probs=probs, loss_t=loss_t)
    return float(loss_t.mean()), stash


def head_bwd(kind: int, stash: Dict[str, np.ndarray], gain: np.ndarray, w: np.ndarray, targets: np.ndarray, v0: int,
             dloss: float = 1.0):
    """Gradient of head_fwd's loss times dloss: (dy [s, b, h], dgain, doffset or None, dW [V_local, h])."""
    hn = stash["hn"]
    s, b, h = hn.shape
    T = s * b
    dlogits = xent_bwd(stash["probs"], np.asarray(targets).reshape(-1), v0, np.full(T, dloss / T))
    dw = dlogits.T @ hn.reshape(T, h)
    dhn = (dlogits @ np.asarray(w, F64)).reshape(s, b, h)
    dy, dgain, doffset = so.norm_bwd(dhn, stash["xhat"], stash["rstd"], np.asarray(gain, F64), kind)
    return dy, dgain, doffset, dw
