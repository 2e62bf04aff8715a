"""AdamW step, float64 numpy -- TEST INFRASTRUCTURE ONLY.

The paper trains the adapter factors with AdamW (Appendix, hyper-parameter tables).
This is Adam with decoupled weight decay, in the convention of the common deep-learning
implementations the paper's setup relies on: the decay multiplies the parameter by
(1 - lr * weight_decay) and is not part of the gradient that enters the moments.

Only the tests may import this module; the GPU library never does.
"""
from __future__ import annotations

import numpy as np


def adamw_step(p, g, m, v, lr, beta1, beta2, eps, weight_decay, step):
    """Returns the updated (p, m, v) as float64 arrays; `step` counts from 1."""
    p = np.asarray(p, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    m_new = beta1 * m + (1.0 - beta1) * g                 # first moment
    v_new = beta2 * v + (1.0 - beta2) * g * g             # second moment
    m_hat = m_new / (1.0 - beta1 ** step)                 # bias corrections
    v_hat = v_new / (1.0 - beta2 ** step)
    p_new = p - lr * weight_decay * p - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p_new, m_new, v_new
