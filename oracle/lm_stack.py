"""fp64 CPU oracle for the rest of the training step around the decoder layers: token
embedding, final RMSNorm, LM head, softmax cross-entropy, and their gradients.

TEST INFRASTRUCTURE ONLY (see oracle/decoder_layer.py for the rules).  The paper shows
only a training-loss curve for its 8B Llama-3-style model (Fig. 2a); the loss itself is
the standard next-token objective, written out here:

  X0[t]   = E[id_t]
  X_l     = layer_l(X_{l-1}),  l = 1..L
  h_f     = RMSNorm(X_L; g_final)
  logits  = h_f W_lm^T                       (untied head)
  loss    = mean_t( logsumexp(logits[t]) - logits[t, target_t] )
  dlogits = (softmax(logits) - onehot(target)) * grad_scale / T

Pinned by tests in `tests/test_oracle_pins.py` (all-zero logits give ln V, gradient rows
sum to zero, shift invariance, finite differences, PyTorch fp64 cross-check).
"""
from __future__ import annotations

import numpy as np

from . import decoder_layer as dl


def ce_loss_fwd_bwd(logits, targets, grad_scale=1.0):
    """logits [T, V] float64, targets [T] int -> (loss scalar, dlogits [T, V], lse [T])."""
    T, V = logits.shape
    m = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - m)
    l = e.sum(axis=-1, keepdims=True)
    lse = (m + np.log(l))[:, 0]
    picked = logits[np.arange(T), targets]
    loss = np.mean(lse - picked)
    dlogits = e / l
    dlogits[np.arange(T), targets] -= 1.0
    dlogits *= grad_scale / T
    return loss, dlogits, lse


def embed_fwd(table, ids):
    """table [V, D], ids [...] -> X0 [..., D]."""
    return table[ids]


def embed_bwd(dx0, ids, vocab):
    """dE[v] = sum over tokens t with id_t == v of dX0[t]."""
    D = dx0.shape[-1]
    dE = np.zeros((vocab, D), dtype=np.float64)
    np.add.at(dE, ids.reshape(-1), dx0.reshape(-1, D))
    return dE


def stack_forward(cfg, ids, targets, embed, layers, g_final, w_lm, row_chunk=1024):
    """Full forward of embedding -> L layers -> final norm -> LM head -> mean CE loss.
    Logits are formed in chunks of rows so the [T, V] fp64 matrix is never held whole."""
    B, S = ids.shape
    D = cfg.d_model
    T = B * S
    st = {"x": [embed_fwd(embed, ids)], "fwd": []}
    for w in layers:
        f = dl.layer_forward(cfg, st["x"][-1], w)
        st["fwd"].append(f)
        st["x"].append(f["y"])
    st["h_f"], st["rstd_f"] = dl.rmsnorm_fwd(st["x"][-1], g_final, cfg.rms_eps)
    hf = st["h_f"].reshape(T, D)
    tg = targets.reshape(T)
    lse = np.empty(T)
    picked = np.empty(T)
    for lo in range(0, T, row_chunk):
        hi = min(T, lo + row_chunk)
        lg = hf[lo:hi] @ w_lm.T
        m = lg.max(axis=-1)
        lse[lo:hi] = m + np.log(np.exp(lg - m[:, None]).sum(axis=-1))
        picked[lo:hi] = lg[np.arange(hi - lo), tg[lo:hi]]
    st["lse"] = lse
    st["loss"] = float(np.mean(lse - picked))
    return st


def stack_backward(cfg, ids, targets, embed, layers, g_final, w_lm, st, grad_scale=1.0,
                   row_chunk=1024):
    """Backward of stack_forward to every parameter and to the input embeddings X0."""
    B, S = ids.shape
    D = cfg.d_model
    T = B * S
    V = w_lm.shape[0]
    hf = st["h_f"].reshape(T, D)
    tg = targets.reshape(T)
    dhf = np.zeros((T, D))
    dw_lm = np.zeros_like(w_lm)
    for lo in range(0, T, row_chunk):
        hi = min(T, lo + row_chunk)
        lg = hf[lo:hi] @ w_lm.T
        p = np.exp(lg - st["lse"][lo:hi, None])
        p[np.arange(hi - lo), tg[lo:hi]] -= 1.0
        p *= grad_scale / T
        dhf[lo:hi] = p @ w_lm
        dw_lm += p.T @ hf[lo:hi]
    g = {"w_lm": dw_lm, "layers": [None] * len(layers)}
    dx, g["g_final"] = dl.rmsnorm_bwd(st["x"][-1], g_final, st["rstd_f"], dhf.reshape(B, S, D))
    for l in reversed(range(len(layers))):
        r = dl.layer_backward(cfg, st["x"][l], layers[l], dx, st["fwd"][l])
        g["layers"][l] = r
        dx = r["dx"]
    g["dx0"] = dx
    g["embed"] = embed_bwd(dx, ids, V)
    return g
