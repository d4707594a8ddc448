"""fp64 CPU oracle for one pre-norm Llama-style causal decoder layer, forward and backward.

TEST INFRASTRUCTURE ONLY.  This file is the plain definition of the layer the paper
benchmarks (its Fig. 2 workload is an 8B Llama-3-style decoder stack; the transformer
block whose per-rank message size it quotes in the Training Pipeline paragraph has
exactly the shape reproduced in `tests/test_oracle_pins.py`).  It is written in NumPy
float64 with explicit S x S attention matrices, no blocking, no fusion and no
re-association, so it can be checked by eye.  It shares no code with the GPU library
and must never be imported by the product path; only tests, the smoke check and the
benchmark's CPU-baseline leg may use it.

The paper gives no equations for the layer; every formula is the standard definition:

  RMSNorm      h = x * rstd * gamma,  rstd = (mean_d x^2 + eps)^(-1/2)
  projections  q = h Wq^T, k = h Wk^T, v = h Wv^T   (weights are [out, in])
  RoPE         pair (a, b) of a head vector at position p rotated by angle
               p * base^(-2i/dh):  a' = a cos - b sin,  b' = a sin + b cos
  attention    o_h = softmax(q_h k_j^T / sqrt(dh) + causal mask) v_j,  j = h // G
  residual     y1 = x + o Wo^T
  SwiGLU MLP   y = y1 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T,  h2 = RMSNorm(y1)

Parity status: every function here is pinned by tests in `tests/test_oracle_pins.py`
(closed forms, invariants, brute force, finite differences, and a stock-PyTorch fp64
autograd cross-check).  The paper prints no worked numerical example for the layer, so
agreement with the authors' own runs is unpinned; only the block's parameter count is
fixed by a number the paper prints.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- RMSNorm
def rmsnorm_fwd(x, gamma, eps):
    """x [..., D], gamma [D] -> (h [..., D], rstd [...])."""
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=-1) + eps)
    return x * rstd[..., None] * gamma, rstd


def rmsnorm_bwd(x, gamma, rstd, dh):
    """Gradient of rmsnorm_fwd: returns (dx [..., D], dgamma [D])."""
    D = x.shape[-1]
    xhat = x * rstd[..., None]
    dgamma = (dh * xhat).reshape(-1, D).sum(axis=0)
    dxhat = dh * gamma
    dx = rstd[..., None] * (dxhat - xhat * np.mean(dxhat * xhat, axis=-1, keepdims=True))
    return dx, dgamma


# ----------------------------------------------------------------------------- RoPE
def rope_angles(seq, head_dim, base):
    """phi[p, i] = p * base^(-2i/head_dim), p = 0..seq-1 (positions restart per sequence)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.power(np.float64(base), -2.0 * i / head_dim)
    return np.arange(seq, dtype=np.float64)[:, None] * theta[None, :]


def rope_rotate(z, phi, layout=0, inverse=False):
    """Rotate head vectors z [B, S, H, dh] by phi [S, dh/2].

    layout 0 pairs element i with i + dh/2; layout 1 pairs 2i with 2i+1.
    inverse=True rotates by -phi, which is the transpose (and so the gradient) of the
    forward rotation.
    """
    c = np.cos(phi)[None, :, None, :]
    s = np.sin(phi)[None, :, None, :]
    if inverse:
        s = -s
    half = z.shape[-1] // 2
    out = np.empty_like(z)
    if layout == 0:
        a, b = z[..., :half], z[..., half:]
        out[..., :half] = a * c - b * s
        out[..., half:] = a * s + b * c
    else:
        a, b = z[..., 0::2], z[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
    return out


# ----------------------------------------------------------------------------- attention
def _causal_probs(qh, kj):
    """Row-softmax of the causally masked, 1/sqrt(dh)-scaled scores. qh, kj: [S, dh]."""
    S, dh = qh.shape
    s = (qh @ kj.T) / np.sqrt(np.float64(dh))
    s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=-1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def attention_fwd(q, k, v):
    """q [B,S,Hq,dh], k, v [B,S,Hkv,dh] (q, k already rotated) -> (o [B,S,Hq,dh], lse [B,Hq,S])."""
    B, S, Hq, dh = q.shape
    G = Hq // k.shape[2]
    o = np.empty_like(q)
    lse = np.empty((B, Hq, S), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            p, lse[b, h] = _causal_probs(q[b, :, h], k[b, :, h // G])
            o[b, :, h] = p @ v[b, :, h // G]
    return o, lse


def attention_bwd(q, k, v, do):
    """Gradients of attention_fwd w.r.t. q, k, v; dK and dV sum over the G query heads of a group."""
    B, S, Hq, dh = q.shape
    G = Hq // k.shape[2]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    scale = 1.0 / np.sqrt(np.float64(dh))
    for b in range(B):
        for h in range(Hq):
            j = h // G
            p, _ = _causal_probs(q[b, :, h], k[b, :, j])
            doh = do[b, :, h]
            dv[b, :, j] += p.T @ doh
            dp = doh @ v[b, :, j].T
            ds = p * (dp - np.sum(p * dp, axis=-1, keepdims=True))
            dq[b, :, h] = (ds @ k[b, :, j]) * scale
            dk[b, :, j] += (ds.T @ q[b, :, h]) * scale
    return dq, dk, dv


# ----------------------------------------------------------------------------- SwiGLU
def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def swiglu_fwd(g, u):
    return g * sigmoid(g) * u


def swiglu_bwd(g, u, da):
    sg = sigmoid(g)
    dg = da * u * sg * (1.0 + g * (1.0 - sg))
    du = da * g * sg
    return dg, du


# ----------------------------------------------------------------------------- whole layer
def layer_forward(cfg, x, w):
    """cfg: object with batch, seq, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, rms_eps,
    rope_base, rope_layout.  x [B,S,D] float64, w: dict of float64 weights ([out, in]).
    Returns a dict holding y and every intermediate tensor."""
    B, S, D = x.shape
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    f = {}
    f["h1"], f["rstd1"] = rmsnorm_fwd(x, w["g_attn"], cfg.rms_eps)
    f["phi"] = rope_angles(S, dh, cfg.rope_base)
    f["q_pre"] = (f["h1"] @ w["wq"].T).reshape(B, S, Hq, dh)
    f["k_pre"] = (f["h1"] @ w["wk"].T).reshape(B, S, Hkv, dh)
    f["v"] = (f["h1"] @ w["wv"].T).reshape(B, S, Hkv, dh)
    f["q"] = rope_rotate(f["q_pre"], f["phi"], cfg.rope_layout)
    f["k"] = rope_rotate(f["k_pre"], f["phi"], cfg.rope_layout)
    f["o"], f["lse"] = attention_fwd(f["q"], f["k"], f["v"])
    f["y1"] = x + f["o"].reshape(B, S, Hq * dh) @ w["wo"].T
    f["h2"], f["rstd2"] = rmsnorm_fwd(f["y1"], w["g_mlp"], cfg.rms_eps)
    f["g"] = f["h2"] @ w["w_gate"].T
    f["u"] = f["h2"] @ w["w_up"].T
    f["a"] = swiglu_fwd(f["g"], f["u"])
    f["y"] = f["y1"] + f["a"] @ w["w_down"].T
    return f


def _linear_bwd(dy2d, x2d, w):
    """y = x W^T  ->  dx = dy W,  dW = dy^T x (sum over all tokens)."""
    return dy2d @ w, dy2d.T @ x2d


def layer_backward(cfg, x, w, dy, f):
    """Hand-derived backward of layer_forward given dL/dy.  Returns dx and the nine weight
    gradients (keys as in w), plus the intermediate gradients."""
    B, S, D = x.shape
    T = B * S
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    F = cfg.d_ff
    r = {}
    # y = y1 + a Wd^T
    da, r["w_down"] = _linear_bwd(dy.reshape(T, D), f["a"].reshape(T, F), w["w_down"])
    r["da"] = da.reshape(B, S, F)
    r["dg"], r["du"] = swiglu_bwd(f["g"], f["u"], r["da"])
    dh2_g, r["w_gate"] = _linear_bwd(r["dg"].reshape(T, F), f["h2"].reshape(T, D), w["w_gate"])
    dh2_u, r["w_up"] = _linear_bwd(r["du"].reshape(T, F), f["h2"].reshape(T, D), w["w_up"])
    r["dh2"] = (dh2_g + dh2_u).reshape(B, S, D)
    dy1_norm, r["g_mlp"] = rmsnorm_bwd(f["y1"], w["g_mlp"], f["rstd2"], r["dh2"])
    r["dy1"] = dy + dy1_norm
    # y1 = x + o Wo^T
    do, r["wo"] = _linear_bwd(r["dy1"].reshape(T, D), f["o"].reshape(T, Hq * dh), w["wo"])
    r["do"] = do.reshape(B, S, Hq, dh)
    r["dq"], r["dk"], r["dv"] = attention_bwd(f["q"], f["k"], f["v"], r["do"])
    r["dq_pre"] = rope_rotate(r["dq"], f["phi"], cfg.rope_layout, inverse=True)
    r["dk_pre"] = rope_rotate(r["dk"], f["phi"], cfg.rope_layout, inverse=True)
    h1 = f["h1"].reshape(T, D)
    dh1_q, r["wq"] = _linear_bwd(r["dq_pre"].reshape(T, Hq * dh), h1, w["wq"])
    dh1_k, r["wk"] = _linear_bwd(r["dk_pre"].reshape(T, Hkv * dh), h1, w["wk"])
    dh1_v, r["wv"] = _linear_bwd(r["dv"].reshape(T, Hkv * dh), h1, w["wv"])
    r["dh1"] = (dh1_q + dh1_k + dh1_v).reshape(B, S, D)
    dx_norm, r["g_attn"] = rmsnorm_bwd(x, w["g_attn"], f["rstd1"], r["dh1"])
    r["dx"] = r["dy1"] + dx_norm
    return r
