"""Why a deep bf16 stack at the 175B-shard width is not held to the one-layer tolerance against an fp64 reference.

CPU only.  The fp64 checker's layer is run twice on the same weights: once on an input drawn in double precision and
once on that input rounded to the bf16 grid, i.e. with the smallest error a bf16 residual stream can carry into a
layer.  The ratio (change of an output tensor) / (change of the input), both in the tests' max-norm metric, is the
layer's amplification of an inherited error.  At hidden 12288 with N(0, 0.02^2) weights the projected queries and
keys have a standard deviation near 2.2 and the scaled attention scores near 5, and the gradients that pass through
the softmax react several times more strongly than the perturbation; at hidden 256, same recipe, the scores are small
and nothing is amplified.  The per-depth tolerances of the full-size GPU tests rest on these two numbers.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import stage_oracle as so


def _metric(a, b):
    return float(np.abs(a - b).max() / np.abs(b).max())


def _amplification(cfg, seed=5):
    p = si.make_layer_params(cfg, 0)
    rng = np.random.Generator(np.random.Philox(key=seed))
    x = rng.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden))            # exact: not on the bf16 grid
    dy = rng.standard_normal((cfg.seq, cfg.micro_batch, cfg.hidden)) * 1e-2
    xr = so.bf16_to_f64(so.bf16_round_nearest_even(x.astype(np.float32))).reshape(x.shape)
    e_in = _metric(xr, x)
    y, st = so.layer_fwd(cfg, p, x)
    dx, g = so.layer_bwd(cfg, p, st, dy)
    score_std = float(np.std(st["q"][:, 0, 0, :] @ st["k"][:, 0, 0, :].T) / np.sqrt(cfg.head_dim))   # head 0, unmasked
    yr, st_r = so.layer_fwd(cfg, p, xr)
    dxr, gr = so.layer_bwd(cfg, p, st_r, dy)
    amp = {"y": _metric(yr, y) / e_in, "dx": _metric(dxr, dx) / e_in}
    for k in g:
        amp[k] = _metric(gr[k], g[k]) / e_in
    return e_in, amp, score_std


def test_input_rounding_is_amplified_at_the_175b_width_and_not_at_a_narrow_one(capsys):
    wide = si.PRESETS["gpt175b"].replace(n_layers=1, seq=160)
    narrow = wide.replace(hidden=256, n_q_heads=2, n_kv_heads=2, ffn=512)
    e_w, amp_w, s_w = _amplification(wide)
    e_n, amp_n, s_n = _amplification(narrow)
    with capsys.disabled():
        print(f"\n  input rounding error (max-norm): wide {e_w:.2e}, narrow {e_n:.2e}; score std {s_w:.2f} / {s_n:.2f}")
        for k in sorted(amp_w, key=lambda k: -amp_w[k]):
            print(f"  amplification {k:14s} hidden 12288: {amp_w[k]:6.2f}   hidden 256: {amp_n.get(k, float('nan')):6.2f}")
    # one bf16 rounding of the input: half a unit in the last place of an 8-bit significand, relative to the largest entry
    assert 1.0e-3 <= e_w <= 2.0 ** -8 and 1.0e-3 <= e_n <= 2.0 ** -8
    assert 3.0 <= s_w <= 7.0 and s_n <= 1.0          # scaled attention scores: about 5 at the wide shape
    # the residual path alone would pass the error through one to one (narrow shape); at the wide shape the attention
    # branch is as large as the residual stream and reacts to the perturbation too
    assert 0.5 <= amp_n["y"] <= 1.5 and 1.2 <= amp_w["y"] <= 2.5
    # ... the gradients of everything below the softmax at the wide shape react several times as strongly
    through_softmax = ("w_qkv", "b_qkv", "norm1_gain", "norm1_offset")
    assert min(amp_w[k] for k in through_softmax) >= 2.0
    assert max(amp_w.values()) <= 12.0
    # at the narrow shape (scores of standard deviation well below 1) nothing is amplified beyond the perturbation
    assert max(amp_n[k] for k in through_softmax) <= 1.5
    assert min(amp_w[k] / amp_n[k] for k in through_softmax) >= 2.0
