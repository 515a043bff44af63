"""CPU oracle for the optimizer step of the LoRA parameters (plain numpy).

TEST INFRASTRUCTURE ONLY, like the rest of ``oracle/``: nothing in the product package may import it.

What the paper fixes (hyperparameter appendix): Adam with beta2 = 0.999, a maximum gradient norm of 0.3, a constant
learning rate (2e-4 up to 13B, 1e-4 for 33B / 65B).  It does not print the update rule; the oracle follows the published
algorithm (Kingma & Ba 2015, Algorithm 1) with bias correction, beta1 = 0.9 and eps = 1e-8 as defaults, weight decay
(off by default) in the decoupled form, and gradient clipping by the global 2-norm in its plain form
g <- g * min(1, c / ||g||).

Every function takes ``dtype``: np.float64 is the definition; np.float32 takes the same steps in the same order with
every operation rounded to fp32, which is the precision the GPU kernel computes in, so that the bf16 copy of the
parameters (a rounding decision) is taken in the same precision on both sides.  Scalars derived from the
hyperparameters (1 - beta, 1 - beta^t, lr * weight_decay, the gradient coefficient) are computed in double precision and
rounded once to ``dtype``.
"""
from __future__ import annotations

import math

import numpy as np


def sqnorm(g) -> float:
    """Sum of squares of a gradient tensor, in double precision."""
    g = np.asarray(g, dtype=np.float64).ravel()
    return float(np.sum(g * g))


def grad_coefficient(sq: float, max_norm: float, grad_scale: float = 1.0) -> float:
    """The factor the accumulated gradient is multiplied by: grad_scale (1 / micro-batches), times the clipping factor
    min(1, max_norm / ||grad_scale * g||) when max_norm > 0.  ``sq`` is sqnorm over ALL parameters' accumulators."""
    if max_norm <= 0.0:
        return float(grad_scale)
    norm = abs(grad_scale) * math.sqrt(sq)
    clip = 1.0 if norm <= max_norm else max_norm / norm
    return float(grad_scale * clip)


def adam_step(p, m, v, g, step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
              weight_decay: float = 0.0, coef: float = 1.0, dtype=np.float64):
    """One Adam step (step = 1 for the first).  Returns new (p, m, v) as arrays of ``dtype``; inputs are not modified.

        g' = coef * g
        m  = beta1 * m + (1 - beta1) * g'
        v  = beta2 * v + (1 - beta2) * g' * g'
        p  = p - lr * weight_decay * p                      (only when weight_decay != 0)
        p  = p - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
    """
    assert step >= 1
    T = np.dtype(dtype).type
    p, m, v, g = (np.array(a, dtype=dtype) for a in (p, m, v, g))
    b1, b2 = T(beta1), T(beta2)
    omb1, omb2 = T(1.0 - beta1), T(1.0 - beta2)
    bc1, bc2 = T(1.0 - beta1 ** step), T(1.0 - beta2 ** step)
    gs = g * T(coef)
    m = b1 * m + omb1 * gs
    v = b2 * v + omb2 * (gs * gs)
    mh = m / bc1
    vh = v / bc2
    d = np.sqrt(vh) + T(eps)
    u = mh / d
    if weight_decay != 0.0:
        p = p - T(lr * weight_decay) * p
    p = p - T(lr) * u
    assert p.dtype == np.dtype(dtype) and m.dtype == p.dtype and v.dtype == p.dtype
    return p, m, v
