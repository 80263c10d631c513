"""Pure-Python loop evaluation of one transformer layer's forward pass and of
one Adam step, for tiny shapes only.

TEST INFRASTRUCTURE ONLY.  It exists to pin the vectorised fp64 checker in
stage_oracle.py: every index is written out as a scalar loop over python
floats (IEEE double) with the `math` module, so a transposed operand, a wrong
head/column mapping or a wrong [seq, batch, hidden] stride in the vectorised
code shows up as a mismatch.  Same layer definition as stage_oracle.py (the
shadow iteration of section 4.2 on a middle-stage partition, section 6.1).
"""
from __future__ import annotations

import math


def _norm_row(row, gain, offset, layernorm, eps):
    h = len(row)
    if layernorm:
        mu = sum(row) / h
        var = sum((t - mu) ** 2 for t in row) / h
        r = 1.0 / math.sqrt(var + eps)
        return [(row[c] - mu) * r * gain[c] + offset[c] for c in range(h)]
    ms = sum(t * t for t in row) / h
    r = 1.0 / math.sqrt(ms + eps)
    return [row[c] * r * gain[c] for c in range(h)]


def _linear_row(row, w, bias):
    """out[o] = sum_c row[c] * w[o][c] (+ bias[o]); w is [out, in]."""
    out = []
    for o in range(len(w)):
        acc = 0.0
        wo = w[o]
        for c in range(len(row)):
            acc += row[c] * wo[c]
        out.append(acc + (bias[o] if bias is not None else 0.0))
    return out


def _gelu(u, erf_form):
    if erf_form:
        return 0.5 * u * (1.0 + math.erf(u / math.sqrt(2.0)))
    return 0.5 * u * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u * u * u)))


def _rotate(vec, pos, theta):
    d = len(vec)
    out = list(vec)
    for j in range(d // 2):
        ang = pos * theta ** (-2.0 * j / d)
        c, s = math.cos(ang), math.sin(ang)
        out[j] = vec[j] * c - vec[j + d // 2] * s
        out[j + d // 2] = vec[j + d // 2] * c + vec[j] * s
    return out


def layer_forward(cfg, p, x):
    """cfg: object with the stage-config attribute names; p: dict of nested
    lists (matrices [out][in], vectors [n]); x: nested list [s][b][h].
    Returns y as nested list [s][b][h]."""
    s, b, h = len(x), len(x[0]), len(x[0][0])
    nq, nkv, d, f = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn
    layernorm = cfg.norm == 0
    A = nq * d
    group = nq // nkv
    bias = (lambda n: p[n]) if cfg.has_bias else (lambda n: None)

    q = [[None] * b for _ in range(s)]
    k = [[None] * b for _ in range(s)]
    v = [[None] * b for _ in range(s)]
    for i in range(s):
        for n in range(b):
            a = _norm_row(x[i][n], p["norm1_gain"], p.get("norm1_offset"), layernorm, cfg.norm_eps)
            qkv = _linear_row(a, p["w_qkv"], bias("b_qkv"))
            qh = [qkv[g * d:(g + 1) * d] for g in range(nq)]
            kh = [qkv[A + g * d:A + (g + 1) * d] for g in range(nkv)]
            vh = [qkv[A + nkv * d + g * d:A + nkv * d + (g + 1) * d] for g in range(nkv)]
            if cfg.pos == 1:
                qh = [_rotate(t, i, cfg.rope_theta) for t in qh]
                kh = [_rotate(t, i, cfg.rope_theta) for t in kh]
            q[i][n], k[i][n], v[i][n] = qh, kh, vh

    y = [[None] * b for _ in range(s)]
    for i in range(s):
        for n in range(b):
            ctx = []
            for g in range(nq):
                kap = g // group
                sc = [sum(q[i][n][g][e] * k[j][n][kap][e] for e in range(d)) / math.sqrt(d) for j in range(i + 1)]
                mx = max(sc)
                ex = [math.exp(t - mx) for t in sc]
                z = sum(ex)
                for e in range(d):
                    ctx.append(sum(ex[j] / z * v[j][n][kap][e] for j in range(i + 1)))
            proj = _linear_row(ctx, p["w_out"], bias("b_out"))
            x1 = [x[i][n][c] + proj[c] for c in range(h)]
            cc = _norm_row(x1, p["norm2_gain"], p.get("norm2_offset"), layernorm, cfg.norm_eps)
            u = _linear_row(cc, p["w_fc1"], bias("b_fc1"))
            if cfg.act == 2:
                g_ = [u[o] / (1.0 + math.exp(-u[o])) * u[f + o] for o in range(f)]
            else:
                g_ = [_gelu(t, cfg.act == 1) for t in u]
            down = _linear_row(g_, p["w_fc2"], bias("b_fc2"))
            y[i][n] = [x1[c] + down[c] for c in range(h)]
    return y


def adam_scalar(p, g, m, v, step, lr, beta1, beta2, eps, weight_decay=0.0, grad_scale=1.0):
    g = grad_scale * g
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    p = p - lr * (mhat / (math.sqrt(vhat) + eps) + weight_decay * p)
    return p, m, v
