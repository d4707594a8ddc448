"""fp64 CPU oracle for the optimizer step that completes the training step: global-norm gradient
clipping followed by AdamW.

TEST INFRASTRUCTURE ONLY (see oracle/decoder_layer.py for the rules): nothing under the product
package may import this module.

The paper's Training Pipeline paragraph speaks of training steps but names no optimizer; the reading
taken is the usual one for this model family, written out from the published definitions:

  clipping (Pascanu et al. 2013, by global norm):
      n = sqrt(sum over all tensors and elements of g^2);  c = min(1, max_norm / (n + 1e-6));  g <- c g
  AdamW (Loshchilov & Hutter 2019, decoupled weight decay; step counter t starts at 1):
      p <- p (1 - lr wd)
      m <- b1 m + (1 - b1) g;      v <- b2 v + (1 - b2) g^2
      p <- p - lr / (1 - b1^t) * m / ( sqrt(v) / sqrt(1 - b2^t) + eps )

The functions work on fp64 arrays; `adamw_step` returns new arrays and leaves its arguments alone.
Storage precision (bf16 parameters and gradients, fp32 moments on the GPU) is the caller's business:
tests round where the method stores.
"""
from __future__ import annotations

import numpy as np

CLIP_EPS = 1e-6


def global_grad_norm(grads) -> float:
    """sqrt of the sum of squares over every element of every tensor in `grads`."""
    return float(np.sqrt(sum(float(np.sum(np.square(np.asarray(g, np.float64)))) for g in grads)))


def clip_coefficient(norm: float, max_norm: float) -> float:
    """Factor the gradients are multiplied by: 1 while the norm is within max_norm."""
    return float(min(1.0, max_norm / (norm + CLIP_EPS)))


def adamw_step(p, g, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, clip_coef=1.0):
    """One AdamW update of one tensor; returns (p_new, m_new, v_new)."""
    p, g, m, v = (np.asarray(a, np.float64) for a in (p, g, m, v))
    g = g * clip_coef
    p_new = p * (1.0 - lr * weight_decay)
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    bc1 = 1.0 - beta1 ** step
    bc2 = 1.0 - beta2 ** step
    p_new = p_new - (lr / bc1) * m_new / (np.sqrt(v_new) / np.sqrt(bc2) + eps)
    return p_new, m_new, v_new
