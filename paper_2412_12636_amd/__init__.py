"""Python binding of libtm_stage.so: argument marshalling only.

Every function has the name and argument order of its C counterpart in
include/tm_stage.h, tm_ops.h, tm_roles.h, tm_sandbox.h and tm_moe.h.  Device tensors are passed either as
integer addresses or as objects with a ``data_ptr()`` method (torch tensors);
this module itself does not import torch.  A non-zero status raises TmError
with the library's message.  There is no fallback: if the shared library is
missing, importing any entry point fails with instructions to build it.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Any, List, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtm_stage.so")

TM_OK, TM_EINVAL, TM_EALIGN, TM_ESIZE, TM_EARCH, TM_ELAUNCH, TM_ESTATE = 0, -1, -2, -3, -4, -5, -6
TM_DTYPE_FP32, TM_DTYPE_BF16 = 0, 1
TM_NORM_LAYERNORM, TM_NORM_RMSNORM = 0, 1
TM_ACT_GELU_TANH, TM_ACT_GELU_ERF, TM_ACT_SWIGLU = 0, 1, 2
TM_POS_NONE, TM_POS_ROTARY = 0, 1
TM_GRAD_ADD, TM_GRAD_STORE, TM_GRAD_TRANSIENT = 0, 1, 2
TM_COMM_PASS, TM_COMM_RECORD, TM_COMM_REPLAY = 0, 1, 2
TM_SCOPE_TP, TM_SCOPE_PP, TM_SCOPE_DP = 1, 2, 4
TM_COLL_ALL_REDUCE, TM_COLL_RECV, TM_COLL_SEND, TM_COLL_BARRIER = 0, 1, 2, 3
(TM_SITE_X, TM_SITE_Y, TM_SITE_DY, TM_SITE_DX, TM_SITE_ATTN_OUT, TM_SITE_MLP_OUT, TM_SITE_D_MLP_IN, TM_SITE_D_ATTN_IN,
 TM_SITE_GRADS, TM_SITE_STEP_END) = range(10)


class TmError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"tm status {code}: {message}")
        self.code = code
        self.message = message


class tm_stage_config_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "seq",
                                         "micro_batch", "dtype", "norm", "act", "pos", "has_bias")] + \
               [("norm_eps", C.c_double), ("rope_theta", C.c_double)]


class tm_stage_buffers_t(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("params", "master", "grads", "exp_avg", "exp_avg_sq", "workspace")] + \
               [("workspace_bytes", C.c_int64)]


class tm_profile_entry_t(C.Structure):
    _fields_ = [("kernel", C.c_char_p), ("ms", C.c_double), ("flops", C.c_double), ("bytes", C.c_double),
                ("launches", C.c_int64)]


class tm_adam_hparams_t(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("lr", "beta1", "beta2", "eps", "weight_decay", "grad_scale")] + \
               [("zero_grads", C.c_int32)]


class tm_moe_config_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tokens", "hidden", "ffn", "n_experts", "ep", "top_k", "capacity", "dtype", "act",
                                         "has_bias")]


TM_MOE_WS_LOGITS, TM_MOE_WS_TOP_IDX, TM_MOE_WS_GATES, TM_MOE_WS_SLOT_ROW = 0, 1, 2, 3


class tm_comm_stats_t(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("calls", "stored", "stored_bytes", "skipped", "native", "tape_entries", "tape_bytes")]


EXPORTS = {
    # name: (restype, argtypes)
    "tm_stage_param_count": (C.c_int64, [C.POINTER(tm_stage_config_t)]),
    "tm_stage_workspace_bytes": (C.c_int64, [C.POINTER(tm_stage_config_t)]),
    "tm_stage_param_layout": (C.c_int, [C.POINTER(tm_stage_config_t), C.c_int, C.POINTER(C.c_char_p),
                                        C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
    "tm_stage_init": (C.c_int, [C.POINTER(tm_stage_config_t), C.POINTER(tm_stage_buffers_t), C.POINTER(C.c_void_p)]),
    "tm_stage_fwd": (C.c_int, [C.c_void_p] * 4),
    "tm_stage_bwd": (C.c_int, [C.c_void_p] * 4),
    "tm_adam_step": (C.c_int, [C.c_void_p, C.POINTER(tm_adam_hparams_t), C.c_int64, C.c_void_p]),
    "tm_stage_grad_sq_sum": (C.c_int, [C.c_void_p] * 3),
    "tm_adam_step_range": (C.c_int, [C.c_void_p, C.c_int64, C.c_int64, C.POINTER(tm_adam_hparams_t), C.c_int64, C.c_void_p]),
    "tm_sq_sum_scratch_bytes": (C.c_int64, [C.c_int64]),
    "tm_sq_sum": (C.c_int, [C.c_int64] + [C.c_void_p] * 4),
    "tm_sq_sum_static_max_elems": (C.c_int64, []),
    "tm_sq_sum_static": (C.c_int, [C.c_int64] + [C.c_void_p] * 3),
    "tm_stage_bwd_adam": (C.c_int, [C.c_void_p] * 3 + [C.POINTER(tm_adam_hparams_t), C.c_int64, C.c_void_p]),
    "tm_adam_step_flat": (C.c_int, [C.c_int64] + [C.c_void_p] * 5 + [C.POINTER(tm_adam_hparams_t), C.c_int64,
                                                                       C.c_void_p]),
    "tm_stage_grad_mode": (C.c_int, [C.c_void_p, C.c_int]),
    "tm_stage_tune": (C.c_int, [C.c_void_p, C.c_void_p]),
    "tm_stage_destroy": (None, [C.c_void_p]),
    "tm_stage_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "tm_stage_profile_collect": (C.c_int, [C.c_void_p, C.POINTER(tm_profile_entry_t), C.c_int]),
    "tm_last_error": (C.c_char_p, []),
    "tm_op_linear_fwd": (C.c_int, [C.c_int] + [C.c_int64] * 3 + [C.c_void_p] * 6),
    "tm_op_linear_dgrad": (C.c_int, [C.c_int] + [C.c_int64] * 3 + [C.c_void_p] * 4),
    "tm_op_linear_dgrad_scratch_bytes": (C.c_int64, [C.c_int] + [C.c_int64] * 3),
    "tm_op_linear_dgrad_ws": (C.c_int, [C.c_int] + [C.c_int64] * 3 + [C.c_void_p] * 4 + [C.c_int64, C.c_void_p]),
    "tm_op_linear_wgrad": (C.c_int, [C.c_int] + [C.c_int64] * 3 + [C.c_void_p] * 3 + [C.c_int, C.c_void_p]),
    "tm_op_reduce_scratch_bytes": (C.c_int64, [C.c_int64, C.c_int64]),
    "tm_op_bias_grad": (C.c_int, [C.c_int, C.c_int64, C.c_int64] + [C.c_void_p] * 3 + [C.c_int, C.c_void_p]),
    "tm_op_norm_fwd": (C.c_int, [C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_double] + [C.c_void_p] * 7),
    "tm_op_norm_bwd": (C.c_int, [C.c_int, C.c_int, C.c_int64, C.c_int64] + [C.c_void_p] * 10 + [C.c_int, C.c_void_p]),
    "tm_op_norm_bwd_colsum": (C.c_int, [C.c_int, C.c_int, C.c_int64, C.c_int64] + [C.c_void_p] * 11 + [C.c_int, C.c_void_p]),
    "tm_op_act_fwd": (C.c_int, [C.c_int, C.c_int, C.c_int64, C.c_int64] + [C.c_void_p] * 3),
    "tm_op_act_bwd": (C.c_int, [C.c_int, C.c_int, C.c_int64, C.c_int64] + [C.c_void_p] * 4),
    "tm_op_rotary": (C.c_int, [C.c_int] + [C.c_int64] * 5 + [C.c_double, C.c_int, C.c_void_p, C.c_void_p]),
    "tm_op_embed_fwd": (C.c_int, [C.c_int] + [C.c_int64] * 5 + [C.c_void_p] * 5),
    "tm_op_embed_bwd": (C.c_int, [C.c_int] + [C.c_int64] * 5 + [C.c_void_p] * 4 + [C.c_int64, C.c_int, C.c_void_p]),
    "tm_op_xent": (C.c_int, [C.c_int] + [C.c_int64] * 3 + [C.c_void_p] * 2 + [C.c_double] + [C.c_void_p] * 3),
    "tm_head_workspace_bytes": (C.c_int64, [C.c_int] + [C.c_int64] * 4),
    "tm_head_fwd_bwd": (C.c_int, [C.c_int, C.c_int, C.c_double] + [C.c_int64] * 5 + [C.c_void_p] * 5 + [C.c_double, C.c_void_p,
                                 C.c_int64] + [C.c_void_p] * 5 + [C.c_int, C.c_void_p]),
    "tm_moe_param_count": (C.c_int64, [C.POINTER(tm_moe_config_t)]),
    "tm_moe_param_layout": (C.c_int, [C.POINTER(tm_moe_config_t), C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_int64),
                                      C.POINTER(C.c_int64)]),
    "tm_moe_workspace_bytes": (C.c_int64, [C.POINTER(tm_moe_config_t)]),
    "tm_moe_workspace_offset": (C.c_int64, [C.POINTER(tm_moe_config_t), C.c_int, C.POINTER(C.c_int64)]),
    "tm_moe_fwd": (C.c_int, [C.POINTER(tm_moe_config_t)] + [C.c_void_p] * 4 + [C.c_int64, C.c_void_p]),
    "tm_moe_bwd": (C.c_int, [C.POINTER(tm_moe_config_t)] + [C.c_void_p] * 5 + [C.c_int, C.c_void_p, C.c_int64, C.c_void_p]),
    "tm_gemm_config_count": (C.c_int, []),
    "tm_gemm_force_config": (C.c_int, [C.c_int]),
    "tm_comm_open": (C.c_int, [C.c_char_p, C.c_int, C.c_int, C.POINTER(C.c_void_p)]),
    "tm_comm_call": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int64, C.c_void_p]),
    "tm_comm_rewind": (C.c_int, [C.c_void_p]),
    "tm_comm_stats": (C.c_int, [C.c_void_p, C.POINTER(tm_comm_stats_t)]),
    "tm_comm_close": (C.c_int, [C.c_void_p]),
    "tm_stage_attach_comm": (C.c_int, [C.c_void_p, C.c_void_p]),
    "tm_stage_grad_sync": (C.c_int, [C.c_void_p, C.c_void_p]),
    "tm_op_bias_residual_add": (C.c_int, [C.c_int, C.c_int64, C.c_int64] + [C.c_void_p] * 5),
    "tm_op_attn_fwd": (C.c_int, [C.c_int] + [C.c_int64] * 5 + [C.c_void_p] * 4),
    "tm_op_attn_bwd_scratch_bytes": (C.c_int64, [C.c_int] + [C.c_int64] * 5),
    "tm_op_attn_bwd": (C.c_int, [C.c_int] + [C.c_int64] * 5 + [C.c_void_p] * 7),
}

_lib = None


def lib() -> C.CDLL:
    """Loads the shared library on first use; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2412_12636_amd.build` "
                              "(hipcc, gfx950); there is no fallback path")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _ptr(t: Any) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _check(status: int) -> int:
    if status < 0:
        raise TmError(int(status), lib().tm_last_error().decode())
    return int(status)


def make_config(cfg: Any) -> tm_stage_config_t:
    """Accepts a tm_stage_config_t or any object with the same attribute names."""
    if isinstance(cfg, tm_stage_config_t):
        return cfg
    out = tm_stage_config_t()
    for name, _ in tm_stage_config_t._fields_:
        setattr(out, name, getattr(cfg, name))
    return out


def make_hparams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0,
                 zero_grads=0) -> tm_adam_hparams_t:
    return tm_adam_hparams_t(lr, beta1, beta2, eps, weight_decay, grad_scale, int(zero_grads))


# ---- tm_stage.h ---------------------------------------------------------------------------------
def tm_stage_param_count(cfg) -> int:
    return _check(lib().tm_stage_param_count(C.byref(make_config(cfg))))


def tm_stage_workspace_bytes(cfg) -> int:
    return _check(lib().tm_stage_workspace_bytes(C.byref(make_config(cfg))))


def tm_stage_param_layout(cfg) -> List[Tuple[str, int, Tuple[int, int]]]:
    """All tensors as (name, element offset, (rows, cols))."""
    c = make_config(cfg)
    n = _check(lib().tm_stage_param_layout(C.byref(c), -1, None, None, None))
    out = []
    for i in range(n):
        name = C.c_char_p()
        off = C.c_int64()
        shape = (C.c_int64 * 2)()
        _check(lib().tm_stage_param_layout(C.byref(c), i, C.byref(name), C.byref(off), shape))
        out.append((name.value.decode(), int(off.value), (int(shape[0]), int(shape[1]))))
    return out


def tm_stage_init(cfg, params, master, grads, exp_avg, exp_avg_sq, workspace, workspace_bytes: Optional[int] = None) -> int:
    """Returns the opaque handle (an integer address).  workspace_bytes: the size of the workspace
    allocation; taken from the tensor when one is passed."""
    if workspace_bytes is None:
        if not hasattr(workspace, "numel"):
            raise ValueError("tm_stage_init: workspace_bytes is required when the workspace is a bare address")
        workspace_bytes = int(workspace.numel()) * int(workspace.element_size())
    b = tm_stage_buffers_t(_ptr(params), _ptr(master), _ptr(grads), _ptr(exp_avg), _ptr(exp_avg_sq), _ptr(workspace),
                           workspace_bytes)
    h = C.c_void_p()
    _check(lib().tm_stage_init(C.byref(make_config(cfg)), C.byref(b), C.byref(h)))
    return h.value


def tm_stage_fwd(handle: int, x_in, y_out, stream: int = 0) -> None:
    _check(lib().tm_stage_fwd(handle, _ptr(x_in), _ptr(y_out), stream))


def tm_stage_bwd(handle: int, dy_in, dx_out, stream: int = 0) -> None:
    _check(lib().tm_stage_bwd(handle, _ptr(dy_in), _ptr(dx_out), stream))


def tm_stage_bwd_adam(handle: int, dy_in, dx_out, hp: tm_adam_hparams_t, step: int, stream: int = 0) -> None:
    _check(lib().tm_stage_bwd_adam(handle, _ptr(dy_in), _ptr(dx_out), C.byref(hp), step, stream))


def tm_stage_grad_sq_sum(handle: int, out, stream: int = 0) -> None:
    _check(lib().tm_stage_grad_sq_sum(handle, _ptr(out), stream))


def tm_adam_step_range(handle: int, first: int, count: int, hp: tm_adam_hparams_t, step: int, stream: int = 0) -> None:
    _check(lib().tm_adam_step_range(handle, first, count, C.byref(hp), step, stream))


def tm_sq_sum_scratch_bytes(n: int) -> int:
    return _check(lib().tm_sq_sum_scratch_bytes(n))


def tm_sq_sum(n: int, g, scratch, out, stream: int = 0) -> None:
    _check(lib().tm_sq_sum(n, _ptr(g), _ptr(scratch), _ptr(out), stream))


def tm_sq_sum_static_max_elems() -> int:
    return int(lib().tm_sq_sum_static_max_elems())


def tm_sq_sum_static(n: int, g, out, stream: int = 0) -> None:
    _check(lib().tm_sq_sum_static(n, _ptr(g), _ptr(out), stream))


def tm_adam_step(handle: int, hp: tm_adam_hparams_t, step: int, stream: int = 0) -> None:
    _check(lib().tm_adam_step(handle, C.byref(hp), step, stream))


def tm_adam_step_flat(n: int, p, g, m, v, p_bf16, hp: tm_adam_hparams_t, step: int, stream: int = 0) -> None:
    _check(lib().tm_adam_step_flat(n, _ptr(p), _ptr(g), _ptr(m), _ptr(v), _ptr(p_bf16), C.byref(hp), step, stream))


def tm_stage_tune(handle: int, stream: int = 0) -> None:
    _check(lib().tm_stage_tune(handle, stream))


def tm_stage_grad_mode(handle: int, mode: int) -> None:
    """mode: TM_GRAD_ADD (0 / False), TM_GRAD_STORE (1 / True), TM_GRAD_TRANSIENT (2)."""
    _check(lib().tm_stage_grad_mode(handle, int(mode)))


def tm_stage_destroy(handle: int) -> None:
    lib().tm_stage_destroy(handle)


def tm_stage_profile_enable(handle: int, enable: bool) -> None:
    _check(lib().tm_stage_profile_enable(handle, int(enable)))


def tm_stage_profile_collect(handle: int, max_entries: int = 64) -> List[dict]:
    """Per-kernel totals since the last collect: kernel, ms, flops, bytes, launches."""
    arr = (tm_profile_entry_t * max_entries)()
    n = _check(lib().tm_stage_profile_collect(handle, arr, max_entries))
    return [dict(kernel=arr[i].kernel.decode(), ms=arr[i].ms, flops=arr[i].flops, bytes=arr[i].bytes,
                 launches=int(arr[i].launches)) for i in range(n)]


def tm_last_error() -> str:
    return lib().tm_last_error().decode()


# ---- tm_ops.h -----------------------------------------------------------------------------------
def tm_op_linear_fwd(dtype, T, N, K, x, w, bias, residual, y, stream=0):
    _check(lib().tm_op_linear_fwd(dtype, T, N, K, _ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), stream))


def tm_op_linear_dgrad(dtype, T, N, K, dy, w, dx, stream=0):
    _check(lib().tm_op_linear_dgrad(dtype, T, N, K, _ptr(dy), _ptr(w), _ptr(dx), stream))


def tm_op_linear_dgrad_scratch_bytes(dtype, T, N, K) -> int:
    return _check(lib().tm_op_linear_dgrad_scratch_bytes(dtype, T, N, K))


def tm_op_linear_dgrad_ws(dtype, T, N, K, dy, w, dx, scratch, scratch_bytes, stream=0):
    _check(lib().tm_op_linear_dgrad_ws(dtype, T, N, K, _ptr(dy), _ptr(w), _ptr(dx), _ptr(scratch), scratch_bytes, stream))


def tm_op_linear_wgrad(dtype, T, N, K, dy, x, dw, accumulate=1, stream=0):
    _check(lib().tm_op_linear_wgrad(dtype, T, N, K, _ptr(dy), _ptr(x), _ptr(dw), int(accumulate), stream))


def tm_op_reduce_scratch_bytes(T, width) -> int:
    return _check(lib().tm_op_reduce_scratch_bytes(T, width))


def tm_op_bias_grad(dtype, T, N, dy, db, scratch, accumulate=1, stream=0):
    _check(lib().tm_op_bias_grad(dtype, T, N, _ptr(dy), _ptr(db), _ptr(scratch), int(accumulate), stream))


def tm_op_norm_fwd(dtype, kind, T, h, eps, x, gain, offset, out, mean, rstd, stream=0):
    _check(lib().tm_op_norm_fwd(dtype, kind, T, h, eps, _ptr(x), _ptr(gain), _ptr(offset), _ptr(out), _ptr(mean),
                                _ptr(rstd), stream))


def tm_op_norm_bwd(dtype, kind, T, h, dout, x, mean, rstd, gain, dres, dx, dgain, doffset, scratch, accumulate=1,
                   stream=0):
    _check(lib().tm_op_norm_bwd(dtype, kind, T, h, _ptr(dout), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gain),
                                _ptr(dres), _ptr(dx), _ptr(dgain), _ptr(doffset), _ptr(scratch), int(accumulate),
                                stream))


def tm_op_act_fwd(dtype, act, T, f, u, g, stream=0):
    _check(lib().tm_op_act_fwd(dtype, act, T, f, _ptr(u), _ptr(g), stream))


def tm_op_act_bwd(dtype, act, T, f, dg, u, du, stream=0):
    _check(lib().tm_op_act_bwd(dtype, act, T, f, _ptr(dg), _ptr(u), _ptr(du), stream))


def tm_op_rotary(dtype, seq, batch, n_heads, d, row_width, theta, inverse, buf, stream=0):
    _check(lib().tm_op_rotary(dtype, seq, batch, n_heads, d, row_width, theta, int(inverse), _ptr(buf), stream))


def tm_op_attn_fwd(dtype, seq, batch, nq, nkv, d, qkv, ctx, lse, stream=0):
    _check(lib().tm_op_attn_fwd(dtype, seq, batch, nq, nkv, d, _ptr(qkv), _ptr(ctx), _ptr(lse), stream))


def tm_op_attn_bwd_scratch_bytes(dtype, seq, batch, nq, nkv, d) -> int:
    return _check(lib().tm_op_attn_bwd_scratch_bytes(dtype, seq, batch, nq, nkv, d))


def tm_op_attn_bwd(dtype, seq, batch, nq, nkv, d, qkv, ctx, dctx, lse, scratch, dqkv, stream=0):
    _check(lib().tm_op_attn_bwd(dtype, seq, batch, nq, nkv, d, _ptr(qkv), _ptr(ctx), _ptr(dctx), _ptr(lse),
                                _ptr(scratch), _ptr(dqkv), stream))


def tm_op_embed_fwd(dtype, seq, batch, h, v_local, v0, tokens, w, pos_emb, x0, stream=0):
    _check(lib().tm_op_embed_fwd(dtype, seq, batch, h, v_local, v0, _ptr(tokens), _ptr(w), _ptr(pos_emb), _ptr(x0), stream))


def tm_op_embed_bwd(dtype, seq, batch, h, v_local, v0, tokens, dx0, dw, dpos, n_pos, accumulate=1, stream=0):
    _check(lib().tm_op_embed_bwd(dtype, seq, batch, h, v_local, v0, _ptr(tokens), _ptr(dx0), _ptr(dw), _ptr(dpos), n_pos,
                                 accumulate, stream))


def tm_op_xent(dtype, T, v_local, v0, logits, targets, dloss, loss_t, loss, stream=0):
    _check(lib().tm_op_xent(dtype, T, v_local, v0, _ptr(logits), _ptr(targets), dloss, _ptr(loss_t), _ptr(loss), stream))


def tm_head_workspace_bytes(dtype, seq, batch, h, v_local) -> int:
    return _check(lib().tm_head_workspace_bytes(dtype, seq, batch, h, v_local))


def tm_head_fwd_bwd(dtype, norm, eps, seq, batch, h, v_local, v0, y, targets, gain, offset, w, dloss, workspace, loss, dy,
                    dgain, doffset, dw, accumulate=1, stream=0, workspace_bytes=None):
    if workspace_bytes is None:
        workspace_bytes = int(workspace.numel()) * int(workspace.element_size())
    _check(lib().tm_head_fwd_bwd(dtype, norm, eps, seq, batch, h, v_local, v0, _ptr(y), _ptr(targets), _ptr(gain), _ptr(offset),
                                 _ptr(w), dloss, _ptr(workspace), workspace_bytes, _ptr(loss), _ptr(dy), _ptr(dgain),
                                 _ptr(doffset), _ptr(dw), accumulate, stream))


def tm_comm_open(path: Optional[str], mode: int, scopes: int) -> int:
    out = C.c_void_p()
    _check(lib().tm_comm_open(None if path is None else os.fsencode(path), mode, scopes, C.byref(out)))
    return int(out.value)


def tm_comm_call(comm: int, kind: int, scope: int, site: int, dtype: int, buf, nbytes: int, stream: int = 0) -> None:
    _check(lib().tm_comm_call(comm, kind, scope, site, dtype, _ptr(buf), nbytes, stream))


def tm_comm_rewind(comm: int) -> None:
    _check(lib().tm_comm_rewind(comm))


def tm_comm_stats(comm: int) -> dict:
    st = tm_comm_stats_t()
    _check(lib().tm_comm_stats(comm, C.byref(st)))
    return {n: int(getattr(st, n)) for n, _ in tm_comm_stats_t._fields_}


def tm_comm_close(comm: int) -> None:
    _check(lib().tm_comm_close(comm))


def tm_stage_attach_comm(handle: int, comm: Optional[int]) -> None:
    _check(lib().tm_stage_attach_comm(handle, comm))


def tm_stage_grad_sync(handle: int, stream: int = 0) -> None:
    _check(lib().tm_stage_grad_sync(handle, stream))


def tm_op_bias_residual_add(dtype, T, h, part, bias, residual, out, stream=0):
    _check(lib().tm_op_bias_residual_add(dtype, T, h, _ptr(part), _ptr(bias), _ptr(residual), _ptr(out), stream))


def tm_gemm_config_count() -> int:
    return _check(lib().tm_gemm_config_count())


def tm_gemm_force_config(index: int) -> None:
    _check(lib().tm_gemm_force_config(index))


def make_moe_config(cfg: Any) -> tm_moe_config_t:
    """From any object with the attribute names of tm_moe_config_t."""
    if isinstance(cfg, tm_moe_config_t):
        return cfg
    return tm_moe_config_t(*[int(getattr(cfg, n)) for n, _ in tm_moe_config_t._fields_])


def tm_moe_param_count(cfg) -> int:
    return _check(lib().tm_moe_param_count(C.byref(make_moe_config(cfg))))


def tm_moe_param_layout(cfg) -> List[Tuple[str, int, Tuple[int, int]]]:
    c = make_moe_config(cfg)
    n = _check(lib().tm_moe_param_layout(C.byref(c), -1, None, None, None))
    out = []
    for i in range(n):
        name, off, shape = C.c_char_p(), C.c_int64(), (C.c_int64 * 2)()
        _check(lib().tm_moe_param_layout(C.byref(c), i, C.byref(name), C.byref(off), shape))
        out.append((name.value.decode(), int(off.value), (int(shape[0]), int(shape[1]))))
    return out


def tm_moe_workspace_bytes(cfg) -> int:
    return _check(lib().tm_moe_workspace_bytes(C.byref(make_moe_config(cfg))))


def tm_moe_workspace_offset(cfg, region: int) -> Tuple[int, int]:
    nbytes = C.c_int64()
    off = _check(lib().tm_moe_workspace_offset(C.byref(make_moe_config(cfg)), region, C.byref(nbytes)))
    return off, int(nbytes.value)


def tm_moe_fwd(cfg, params, c, out, workspace, stream: int = 0, workspace_bytes: Optional[int] = None) -> None:
    if workspace_bytes is None:
        workspace_bytes = int(workspace.numel()) * int(workspace.element_size())
    _check(lib().tm_moe_fwd(C.byref(make_moe_config(cfg)), _ptr(params), _ptr(c), _ptr(out), _ptr(workspace), workspace_bytes, stream))


def tm_moe_bwd(cfg, params, c, dout, dc, grads, accumulate, workspace, stream: int = 0, workspace_bytes: Optional[int] = None) -> None:
    if workspace_bytes is None:
        workspace_bytes = int(workspace.numel()) * int(workspace.element_size())
    _check(lib().tm_moe_bwd(C.byref(make_moe_config(cfg)), _ptr(params), _ptr(c), _ptr(dout), _ptr(dc), _ptr(grads), accumulate,
                            _ptr(workspace), workspace_bytes, stream))


def tm_op_norm_bwd_colsum(dtype, kind, T, h, dout, x, mean, rstd, gain, dres, dx, dgain, doffset, dx_colsum, scratch,
                          accumulate=1, stream=0):
    _check(lib().tm_op_norm_bwd_colsum(dtype, kind, T, h, _ptr(dout), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gain), _ptr(dres),
                                       _ptr(dx), _ptr(dgain), _ptr(doffset), _ptr(dx_colsum), _ptr(scratch), accumulate, stream))
