"""ctypes binding for libdlayer.so.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_PKG, "libdlayer.so")

WEIGHT_FIELDS = ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")

EXPORTED_SYMBOLS = (
    "dlayer_version", "dlayer_last_error", "dlayer_saved_bytes", "dlayer_workspace_bytes",
    "dlayer_forward", "dlayer_backward", "ce_loss_workspace_bytes", "ce_loss_fwd_bwd", "ce_loss_fwd_bwd_static",
    "lm_head_ce_workspace_bytes", "lm_head_ce_fwd_bwd",
    "rmsnorm_forward", "rmsnorm_backward_workspace_bytes", "rmsnorm_backward",
    "linear_forward", "qkv_rope_workspace_bytes", "qkv_rope_forward", "linear_swiglu_forward", "linear_swiglu_backward_workspace_bytes",
    "linear_swiglu_backward", "linear_backward_workspace_bytes", "linear_backward", "linear_wgrad_group", "rope_apply",
    "attention_forward", "attention_backward_workspace_bytes", "attention_backward",
    "swiglu_forward", "swiglu_backward", "embed_forward", "embed_backward_workspace_bytes", "embed_backward",
    "grad_sq_norm_workspace_bytes", "grad_sq_norm", "adamw_step", "issue_rate_probe",
)


DLAYER_ACCUMULATE_WGRADS = 1
DLAYER_REUSE_TRANSPOSED_WEIGHTS = 2
DLAYER_RECOMPUTE_NORMS = 1
DLAYER_RECOMPUTE_SWIGLU = 2


class DLayerError(RuntimeError):
    pass


class LayerCfg(C.Structure):
    """Mirror of `dlayer_cfg`."""
    _fields_ = [("batch", C.c_int32), ("seq", C.c_int32), ("d_model", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ff", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("rope_layout", C.c_int32), ("recompute", C.c_int32)]

    @classmethod
    def of(cls, cfg) -> "LayerCfg":
        """Accepts a LayerCfg or any object with the same attribute names."""
        if isinstance(cfg, cls):
            return cfg
        return cls(*(getattr(cfg, n, 0) for n, _ in cls._fields_))


class _Ptrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


def _load():
    if not os.path.exists(lib_path):
        raise DLayerError(
            f"{lib_path} is missing: build it first (python -m paper_2602_08387_amd.build); "
            "there is no fallback implementation")
    l = C.CDLL(lib_path)
    vp, i64, sz, i32, f32 = C.c_void_p, C.c_int64, C.c_size_t, C.c_int32, C.c_float
    cfgp = C.POINTER(LayerCfg)
    ptrs = C.POINTER(_Ptrs)
    sig = {
        "dlayer_version": (C.c_int, []),
        "dlayer_last_error": (C.c_char_p, []),
        "dlayer_saved_bytes": (sz, [cfgp]),
        "dlayer_workspace_bytes": (sz, [cfgp]),
        "dlayer_forward": (C.c_int, [cfgp, vp, ptrs, vp, vp, vp, vp]),
        "dlayer_backward": (C.c_int, [cfgp, vp, ptrs, vp, vp, vp, ptrs, C.c_int, vp, vp]),
        "ce_loss_workspace_bytes": (sz, [i64, i64]),
        "lm_head_ce_workspace_bytes": (sz, [i64, i64, i64, i64]),
        "lm_head_ce_fwd_bwd": (C.c_int, [vp, vp, vp, i64, i64, i64, C.c_float, i64, vp, vp, vp, C.c_int, vp, vp]),
        "ce_loss_fwd_bwd": (C.c_int, [vp, vp, i64, i64, f32, vp, vp, vp, vp]),
        "ce_loss_fwd_bwd_static": (C.c_int, [vp, vp, i64, i64, f32, vp, vp, vp]),
        "rmsnorm_forward": (C.c_int, [vp, vp, i64, i64, f32, vp, vp, vp]),
        "rmsnorm_backward_workspace_bytes": (sz, [i64, i64]),
        "rmsnorm_backward": (C.c_int, [vp, vp, vp, vp, vp, i64, i64, vp, vp, C.c_int, vp, vp]),
        "linear_forward": (C.c_int, [vp, vp, vp, i64, i64, i64, vp, vp]),
        "qkv_rope_workspace_bytes": (sz, [i64, i64]),
        "qkv_rope_forward": (C.c_int, [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, f32, i32, vp, vp, vp, vp, vp]),
        "linear_swiglu_forward": (C.c_int, [vp, vp, vp, i64, i64, i64, vp, vp, vp, vp]),
        "linear_swiglu_backward_workspace_bytes": (C.c_size_t, [i64, i64, i64]),
        "linear_swiglu_backward": (C.c_int, [vp, vp, vp, vp, i64, i64, i64, vp, vp, vp, vp]),
        "linear_backward_workspace_bytes": (sz, [i64, i64, i64]),
        "linear_backward": (C.c_int, [vp, vp, vp, i64, i64, i64, vp, vp, C.c_int, vp, vp]),
        "linear_wgrad_group": (C.c_int, [i32, vp, vp, vp, vp, i64, vp, C.c_int, vp]),
        "rope_apply": (C.c_int, [vp, i64, i64, i64, i64, f32, i32, i32, vp]),
        "attention_forward": (C.c_int, [vp, vp, vp, i64, i64, i64, i64, i64, vp, vp, vp]),
        "attention_backward_workspace_bytes": (sz, [i64, i64, i64, i64, i64]),
        "attention_backward": (C.c_int, [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, vp, vp, vp, vp, vp]),
        "swiglu_forward": (C.c_int, [vp, vp, i64, vp, vp]),
        "swiglu_backward": (C.c_int, [vp, vp, vp, i64, vp, vp, vp]),
        "embed_forward": (C.c_int, [vp, vp, i64, i64, i64, vp, vp]),
        "embed_backward_workspace_bytes": (sz, [i64, i64]),
        "embed_backward": (C.c_int, [vp, vp, i64, i64, i64, vp, vp, vp]),
        "grad_sq_norm_workspace_bytes": (sz, [i32, vp]),
        "grad_sq_norm": (C.c_int, [i32, vp, vp, vp, C.c_int, vp, vp]),
        "adamw_step": (C.c_int, [i32, vp, vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, f32, vp, vp]),
        "issue_rate_probe": (C.c_int, [C.c_int, C.c_int, C.c_int, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(l, name)
        fn.restype = res
        fn.argtypes = args
    return l


lib = _load()


def _p(t):
    """Device pointer of a torch tensor (or None -> NULL).  Tensors must be contiguous."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise DLayerError("tensor arguments must be contiguous")
    if not t.is_cuda:
        raise DLayerError("tensor arguments must live on the GPU")
    return t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc, name):
    if rc != 0:
        raise DLayerError(f"{name} failed with status {rc}: {lib.dlayer_last_error().decode()}")


def _ptr_struct(d):
    return _Ptrs(*(_p(d[n]) for n in WEIGHT_FIELDS))


def dlayer_version() -> int:
    return lib.dlayer_version()


def dlayer_saved_bytes(cfg) -> int:
    return lib.dlayer_saved_bytes(C.byref(LayerCfg.of(cfg)))


def dlayer_workspace_bytes(cfg) -> int:
    return lib.dlayer_workspace_bytes(C.byref(LayerCfg.of(cfg)))


def dlayer_forward(cfg, x, weights, y, saved, workspace, stream=None):
    _check(lib.dlayer_forward(C.byref(LayerCfg.of(cfg)), _p(x), C.byref(_ptr_struct(weights)), _p(y),
                              _p(saved), _p(workspace), _stream(stream)), "dlayer_forward")


def dlayer_backward(cfg, x, weights, dy, saved, dx, wgrads, flags, workspace, stream=None):
    _check(lib.dlayer_backward(C.byref(LayerCfg.of(cfg)), _p(x), C.byref(_ptr_struct(weights)), _p(dy),
                               _p(saved), _p(dx), C.byref(_ptr_struct(wgrads)), int(flags),
                               _p(workspace), _stream(stream)), "dlayer_backward")


def ce_loss_workspace_bytes(T, V) -> int:
    return lib.ce_loss_workspace_bytes(T, V)


def lm_head_ce_workspace_bytes(T, D, V, chunk_rows=0) -> int:
    return lib.lm_head_ce_workspace_bytes(T, D, V, chunk_rows)


def lm_head_ce_fwd_bwd(h, w_lm, targets, T, D, V, grad_scale, chunk_rows, loss, dh, dw_lm, accumulate_dw, workspace,
                       stream=None):
    _check(lib.lm_head_ce_fwd_bwd(_p(h), _p(w_lm), _p(targets), T, D, V, grad_scale, chunk_rows, _p(loss), _p(dh),
                                  _p(dw_lm), int(accumulate_dw), _p(workspace), _stream(stream)), "lm_head_ce_fwd_bwd")


def ce_loss_fwd_bwd(logits, targets, T, V, grad_scale, loss, dlogits, workspace, stream=None):
    _check(lib.ce_loss_fwd_bwd(_p(logits), _p(targets), T, V, grad_scale, _p(loss), _p(dlogits),
                               _p(workspace), _stream(stream)), "ce_loss_fwd_bwd")


def ce_loss_fwd_bwd_static(logits, targets, T, V, grad_scale, loss, dlogits, stream=None):
    _check(lib.ce_loss_fwd_bwd_static(_p(logits), _p(targets), T, V, grad_scale, _p(loss), _p(dlogits),
                                      _stream(stream)), "ce_loss_fwd_bwd_static")


def rmsnorm_forward(x, gamma, T, D, eps, h, rstd, stream=None):
    _check(lib.rmsnorm_forward(_p(x), _p(gamma), T, D, eps, _p(h), _p(rstd), _stream(stream)),
           "rmsnorm_forward")


def rmsnorm_backward_workspace_bytes(T, D) -> int:
    return lib.rmsnorm_backward_workspace_bytes(T, D)


def rmsnorm_backward(x, gamma, rstd, dh, dres, T, D, dx, dgamma, accumulate_dgamma, workspace, stream=None):
    _check(lib.rmsnorm_backward(_p(x), _p(gamma), _p(rstd), _p(dh), _p(dres), T, D, _p(dx), _p(dgamma),
                                int(accumulate_dgamma), _p(workspace), _stream(stream)), "rmsnorm_backward")


def linear_forward(x, w, residual, T, K, N, y, stream=None):
    _check(lib.linear_forward(_p(x), _p(w), _p(residual), T, K, N, _p(y), _stream(stream)), "linear_forward")


def linear_backward_workspace_bytes(T, K, N) -> int:
    return lib.linear_backward_workspace_bytes(T, K, N)


def linear_backward(x, w, dy, T, K, N, dx, dw, accumulate_dw, workspace, stream=None):
    _check(lib.linear_backward(_p(x), _p(w), _p(dy), T, K, N, _p(dx), _p(dw), int(accumulate_dw),
                               _p(workspace), _stream(stream)), "linear_backward")


def qkv_rope_workspace_bytes(seq, head_dim) -> int:
    return lib.qkv_rope_workspace_bytes(seq, head_dim)


def qkv_rope_forward(h, wq, wk, wv, batch, seq, d_model, n_q_heads, n_kv_heads, head_dim, rope_base, rope_layout,
                     q, k, v, workspace, stream=None):
    _check(lib.qkv_rope_forward(_p(h), _p(wq), _p(wk), _p(wv), batch, seq, d_model, n_q_heads, n_kv_heads, head_dim,
                                rope_base, rope_layout, _p(q), _p(k), _p(v), _p(workspace), _stream(stream)),
           "qkv_rope_forward")


def linear_swiglu_forward(x, w_gate, w_up, T, K, F, g, u, a, stream=None):
    _check(lib.linear_swiglu_forward(_p(x), _p(w_gate), _p(w_up), T, K, F, _p(g), _p(u), _p(a), _stream(stream)),
           "linear_swiglu_forward")


def linear_swiglu_backward_workspace_bytes(T, D, F) -> int:
    return lib.linear_swiglu_backward_workspace_bytes(T, D, F)


def linear_swiglu_backward(dy, w_down, g, u, T, D, F, dg, du, workspace, stream=None):
    _check(lib.linear_swiglu_backward(_p(dy), _p(w_down), _p(g), _p(u), T, D, F, _p(dg), _p(du), _p(workspace),
                                      _stream(stream)), "linear_swiglu_backward")


def linear_wgrad_group(dys, xs, Ns, Ks, T, dws, accumulate_dw, stream=None):
    n = len(dys)
    assert len(xs) == len(Ns) == len(Ks) == len(dws) == n
    ptrs = lambda ts: (C.c_void_p * n)(*[_p(t) for t in ts])
    i64s = lambda vs: (C.c_int64 * n)(*[int(v) for v in vs])
    _check(lib.linear_wgrad_group(n, ptrs(dys), ptrs(xs), i64s(Ns), i64s(Ks), T, ptrs(dws), int(accumulate_dw),
                                  _stream(stream)), "linear_wgrad_group")


def rope_apply(z, batch, seq, n_heads, head_dim, rope_base, rope_layout, inverse, stream=None):
    _check(lib.rope_apply(_p(z), batch, seq, n_heads, head_dim, rope_base, rope_layout, int(inverse),
                          _stream(stream)), "rope_apply")


def attention_forward(q, k, v, batch, seq, n_q_heads, n_kv_heads, head_dim, o, lse, stream=None):
    _check(lib.attention_forward(_p(q), _p(k), _p(v), batch, seq, n_q_heads, n_kv_heads, head_dim, _p(o),
                                 _p(lse), _stream(stream)), "attention_forward")


def attention_backward_workspace_bytes(batch, seq, n_q_heads, n_kv_heads, head_dim) -> int:
    return lib.attention_backward_workspace_bytes(batch, seq, n_q_heads, n_kv_heads, head_dim)


def attention_backward(q, k, v, o, d_o, lse, batch, seq, n_q_heads, n_kv_heads, head_dim, dq, dk, dv,
                       workspace, stream=None):
    _check(lib.attention_backward(_p(q), _p(k), _p(v), _p(o), _p(d_o), _p(lse), batch, seq, n_q_heads,
                                  n_kv_heads, head_dim, _p(dq), _p(dk), _p(dv), _p(workspace),
                                  _stream(stream)), "attention_backward")


def swiglu_forward(g, u, n, a, stream=None):
    _check(lib.swiglu_forward(_p(g), _p(u), n, _p(a), _stream(stream)), "swiglu_forward")


def swiglu_backward(g, u, da, n, dg, du, stream=None):
    _check(lib.swiglu_backward(_p(g), _p(u), _p(da), n, _p(dg), _p(du), _stream(stream)), "swiglu_backward")


def embed_forward(table, ids, T, V, D, x0, stream=None):
    _check(lib.embed_forward(_p(table), _p(ids), T, V, D, _p(x0), _stream(stream)), "embed_forward")


def embed_backward_workspace_bytes(T, V) -> int:
    return lib.embed_backward_workspace_bytes(T, V)


def embed_backward(dx0, ids, T, V, D, dtable, workspace, stream=None):
    _check(lib.embed_backward(_p(dx0), _p(ids), T, V, D, _p(dtable), _p(workspace), _stream(stream)), "embed_backward")


def _ptr_list(ts):
    return (C.c_void_p * len(ts))(*[_p(t) for t in ts])


def _numel_list(ts):
    return (C.c_int64 * len(ts))(*[int(t.numel()) for t in ts])


def grad_sq_norm_workspace_bytes(grads) -> int:
    return lib.grad_sq_norm_workspace_bytes(len(grads), _numel_list(grads))


def grad_sq_norm(grads, sq_norm, accumulate, workspace, stream=None):
    _check(lib.grad_sq_norm(len(grads), _ptr_list(grads), _numel_list(grads), _p(sq_norm), int(accumulate),
                            _p(workspace), _stream(stream)), "grad_sq_norm")


def adamw_step(params, grads, exp_avg, exp_avg_sq, step, lr, beta1, beta2, eps, weight_decay, max_grad_norm,
               sq_norm, stream=None):
    n = len(params)
    assert len(grads) == len(exp_avg) == len(exp_avg_sq) == n
    _check(lib.adamw_step(n, _ptr_list(params), _ptr_list(grads), _ptr_list(exp_avg), _ptr_list(exp_avg_sq),
                          _numel_list(params), int(step), lr, beta1, beta2, eps, weight_decay, max_grad_norm,
                          _p(sq_norm), _stream(stream)), "adamw_step")


def issue_rate_probe(family, variant, waves_per_simd=2, stream=None):
    """(cycles per block per SIMD, milliseconds, shader clock in GHz, second role's cycles per op)"""
    out = (C.c_double * 4)()
    _check(lib.issue_rate_probe(family, variant, waves_per_simd, out, _stream(stream)), "issue_rate_probe")
    return tuple(out)
