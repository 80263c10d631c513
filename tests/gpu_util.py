"""Helpers of the GPU parity tests: device buffers (torch is used for memory only), dtype
conversion, and the error metric.

Error metric: for a tensor with reference values b and computed values a,
    err = max_i |a_i - b_i| / max_i |b_i|
(an elementwise relative error does not exist for N(0, sigma) data with entries near zero).
Beside it the tests report pass_rate(): the share of elements within rtol*|b| + rtol*rms(b).
Tolerances: bf16 activations and gradients 2e-2; fp32 stages 1e-4 (fp32 accumulation over at
most a few thousand terms: ~1e-6 per operation, chained through two layers); fp32 master weights
after Adam 1e-5.
"""
from __future__ import annotations

import numpy as np
import pytest

import synth_inputs as si

TOL_BF16 = 2e-2
TOL_FP32 = 1e-4
TOL_ADAM = 1e-5


def require_gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def torch_dtype(torch, dtype: int):
    return torch.bfloat16 if dtype == si.DTYPE_BF16 else torch.float32


def to_dev(torch, a: np.ndarray, dtype: int):
    """Host fp32/fp64 array -> device tensor of the stage dtype.  bf16: the values must already
    lie on the bf16 grid (the conversion is then exact)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    t = torch.from_numpy(a32).cuda()
    if dtype == si.DTYPE_BF16:
        tb = t.to(torch.bfloat16)
        assert bool((tb.float() == t).all()), "input is not bf16-exact"
        return tb
    return t


def f32_dev(torch, a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(a: np.ndarray, b: np.ndarray) -> float:
    a = np.asarray(a, np.float64).reshape(-1)
    b = np.asarray(b, np.float64).reshape(-1)
    assert a.shape == b.shape, (a.shape, b.shape)
    assert np.isfinite(a).all(), "non-finite values in the GPU result"
    den = np.abs(b).max()
    return float(np.abs(a - b).max() / (den if den > 0 else 1.0))


def pass_rate(a: np.ndarray, b: np.ndarray, rtol: float) -> float:
    """Share of the elements with |a - b| <= rtol * |b| + rtol * rms(b): the elementwise companion of rel_err (an
    element near zero is held to rtol of the tensor's typical size, a large one to rtol of itself)."""
    a = np.asarray(a, np.float64).reshape(-1)
    b = np.asarray(b, np.float64).reshape(-1)
    assert a.shape == b.shape, (a.shape, b.shape)
    rms = float(np.sqrt(np.mean(b * b)))
    return float(np.mean(np.abs(a - b) <= rtol * np.abs(b) + rtol * rms))


def snap(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return si.snap_to_bf16_grid(a) if dtype == si.DTYPE_BF16 else a


def rand(rng, shape, std, dtype, mean=0.0):
    return snap((rng.standard_normal(shape) * std + mean).astype(np.float32), dtype)


def stream_ptr(torch) -> int:
    return int(torch.cuda.current_stream().cuda_stream)
