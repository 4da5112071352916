"""Float64 reference of the decoupled-weight-decay Adam update.

TEST INFRASTRUCTURE ONLY (see oracle/model.py).  The paper's Section 4.1
gives only learning-rate range and schedule; the update rule is the
standard AdamW one, with the decay term using the weight before the step:

  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
  w <- w - lr * ( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + wd * w )
"""
import numpy as np


def adamw_update(w, g, m, v, step, lr, beta1, beta2, eps, weight_decay):
    """All float64 arrays; ``step`` counts from 1.  Returns (w, m, v)."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    w_new = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    return w_new, m, v


def cosine_lr(step, total_steps, peak_lr, warmup_frac=0.05):
    """Cosine schedule with linear warm-up (Section 4.1: 5 % warm-up).
    ``step`` counts from 0."""
    warm = max(1, int(round(warmup_frac * total_steps)))
    if step < warm:
        return peak_lr * (step + 1) / warm
    prog = (step - warm) / max(1, total_steps - warm)
    return 0.5 * peak_lr * (1.0 + np.cos(np.pi * min(1.0, prog)))
