"""Plain fp64 CPU oracle for the AdamW step used beside Muon for non-matrix parameters.

TEST INFRASTRUCTURE ONLY (never imported by the product package; shares no code with the HIP path).

Section 2.2 ("Matching update RMS of AdamW") states that RMSNorm gains, the LM head and the embeddings stay on
AdamW and share the learning rate and weight decay with Muon; the paper does not restate AdamW, so this is the
published algorithm (Adam with bias correction, Kingma & Ba; decoupled weight decay, Loshchilov & Hutter),
written out term by term:

    m_t = beta1 m_{t-1} + (1 - beta1) g
    v_t = beta2 v_{t-1} + (1 - beta2) g^2
    mhat = m_t / (1 - beta1^t),  vhat = v_t / (1 - beta2^t)
    p_t = p_{t-1} - lr * (mhat / (sqrt(vhat) + eps) + weight_decay * p_{t-1})

Pinned by pure-Python loops, the constant-gradient closed form (mhat = g and vhat = g^2 at every step), and
degenerate settings.  Nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def adamw_step(p, g, m, v, *, lr: float, weight_decay: float, beta1: float = 0.9, beta2: float = 0.95,
               eps: float = 1e-8, step: int = 1):
    """One AdamW step (step counts from 1).  Returns (p_t, m_t, v_t) in float64."""
    if int(step) < 1:
        raise ValueError("step counts from 1")
    p = np.asarray(p, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m = float(beta1) * np.asarray(m, dtype=np.float64) + (1.0 - float(beta1)) * g
    v = float(beta2) * np.asarray(v, dtype=np.float64) + (1.0 - float(beta2)) * g * g
    mhat = m / (1.0 - float(beta1) ** int(step))
    vhat = v / (1.0 - float(beta2) ** int(step))
    p_new = p - float(lr) * (mhat / (np.sqrt(vhat) + float(eps)) + float(weight_decay) * p)
    return p_new, m, v
