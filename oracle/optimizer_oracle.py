"""CPU oracle for the parameter update that follows gradient accumulation.

TEST INFRASTRUCTURE ONLY.  Plain float64 numpy; shares nothing with the HIP library.

The paper's training step ends with `state.apply_gradient(grads, learning_rate)` (Section
3.1) and does not say which optimizer; the two rules below are the published ones, stated
per element:

  SGD with L2 term:   w <- w - lr * (g + wd * w)
  AdamW (decoupled weight decay, bias-corrected moments), step t = 1, 2, ...:
      m <- b1 m + (1 - b1) g;   v <- b2 v + (1 - b2) g^2
      mhat = m / (1 - b1^t);    vhat = v / (1 - b2^t)
      w <- w - lr * (mhat / (sqrt(vhat) + eps) + wd * w)

Pinned in tests/test_optimizer_oracle_pins.py against closed forms and against an independent
library implementation of both rules.
"""
import numpy as np


def sgd_step(w, g, lr, weight_decay=0.0):
    return w - lr * (g + weight_decay * w)


def adamw_step(w, m, v, g, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """Returns (w, m, v) after step t (1-based)."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    w = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    return w, m, v
