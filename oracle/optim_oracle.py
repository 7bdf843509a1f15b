"""CPU checker for the update that closes an iteration (test infrastructure, never the product path).

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg import this.

The paper's convergence runs (appendix "Test Configurations") fix two things about the update: the
learning rate, 3e-4, and that gradient norms are clipped to 1.0.  It does not name the optimiser; the
reading taken here is AdamW (decoupled weight decay), the usual choice for the LLaMa family it trains,
with the update written out from its published definition:

    g      <- g * min(1, clip / (||g||_2 + 1e-6))          one norm over all parameters of the call
    m      <- b1 m + (1 - b1) g
    v      <- b2 v + (1 - b2) g^2
    p      <- p (1 - lr wd) - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)

in float64, plain numpy, one array operation per line of the definition.  Pins (tests/test_oracle_optim.py):
the library routines ``torch.optim.AdamW`` + ``torch.nn.utils.clip_grad_norm_`` over several steps, the
closed form of the first step (a step of lr against the sign of the gradient), the clip invariants and the
pure-decay case.
"""
from __future__ import annotations

import numpy as np

PAPER_LR = 3e-4        # appendix "Test Configurations"
PAPER_CLIP = 1.0       # appendix "Test Configurations"


def clip_coefficient(grads: np.ndarray, clip: float) -> tuple[float, float]:
    """(total 2-norm of grads, factor that scales it to at most clip); clip <= 0 means no clipping."""
    g = np.asarray(grads, np.float64).reshape(-1)
    norm = float(np.sqrt(np.sum(g * g)))
    if clip <= 0:
        return norm, 1.0
    return norm, min(1.0, clip / (norm + 1e-6))


def adamw_step(p, g, m, v, step: int, lr: float = PAPER_LR, beta1: float = 0.9, beta2: float = 0.999,
               eps: float = 1e-8, weight_decay: float = 0.01, clip: float = PAPER_CLIP):
    """One update of all parameters p (any shape) with gradients g and moments m, v; step counts from 1.

    Returns (p_new, m_new, v_new, grad_norm) as float64 arrays; inputs are not modified.
    """
    p = np.asarray(p, np.float64); g = np.asarray(g, np.float64)
    m = np.asarray(m, np.float64); v = np.asarray(v, np.float64)
    norm, coef = clip_coefficient(g, clip)
    g = g * coef
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m_new / (1.0 - beta1 ** step)
    v_hat = v_new / (1.0 - beta2 ** step)
    p_new = p * (1.0 - lr * weight_decay) - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p_new, m_new, v_new, norm
