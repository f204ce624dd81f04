"""AdamW update of a flat parameter buffer (test infrastructure; see the package docstring). float64.

The paper names the optimiser (AdamW) and its learning rate (1e-3) in section "Numerical Results", paragraph on the
training setup, and gives nothing else, so the update is the published algorithm (Adam with decoupled weight
decay, Loshchilov & Hutter) and the remaining constants are this build's reading: beta1 = 0.9, beta2 = 0.999,
eps = 1e-8, decay 0.01 (what the common implementations default to).

  m <- beta1 m + (1 - beta1) g
  v <- beta2 v + (1 - beta2) g*g
  mhat = m / (1 - beta1^t),  vhat = v / (1 - beta2^t)          t = 1, 2, ... counts the updates
  w <- w - lr * ( mhat / (sqrt(vhat) + eps) + decay * w )       (the decay acts on w before the update)

Pins (tests/test_oracle_optim.py): torch.optim.AdamW on float64 tensors over several steps, the closed form of
the first step from zero moments, pure decay when every gradient is zero, invariance to the gradient scale.
"""
from __future__ import annotations

import numpy as np

DEFAULTS = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def adamw_step(w, g, m, v, t, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """One update number t (>= 1). Returns new (w, m, v); inputs are not modified."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    w_new = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    return w_new, m, v
