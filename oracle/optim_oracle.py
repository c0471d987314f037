"""CPU oracle for the optimizer step the paper trains the layer's parameters {A, B, scale, zero} with
(App. C "Experimental Settings": AdamW with weight decay 0.01, cosine decay with linear warm-up over the
first 10 % of the steps).  TEST INFRASTRUCTURE ONLY; shares no code with the HIP path.

The paper gives neither betas nor epsilon nor the end value of the cosine: read as the common defaults
beta1 = 0.9, beta2 = 0.999, eps = 1e-8, decay to zero.  Decoupled weight decay as in the AdamW paper:
    m <- b1 m + (1 - b1) g;  v <- b2 v + (1 - b2) g^2
    p <- p - lr * wd * p - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),   t = 1, 2, ...
Pins (tests/test_oracle_optim.py): first-step closed form, constant-gradient fixed point of the bias
correction, and torch.optim.AdamW on the CPU as an independent library routine.
"""
from __future__ import annotations

import math

import numpy as np


def adamw_step(p, g, m, v, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1):
    """One AdamW update in float64.  Returns (p, m, v) as new arrays; `step` counts from 1."""
    p, g, m, v = (np.asarray(a, np.float64) for a in (p, g, m, v))
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    p = p - lr * weight_decay * p - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


def cosine_lr(step: int, total_steps: int, lr_max: float, warmup_fraction: float = 0.1) -> float:
    """Learning rate of 0-based `step`: linear warm-up lr_max (step + 1) / W over the first
    W = ceil(warmup_fraction * total_steps) steps, then half a cosine from lr_max down to 0 at total_steps."""
    w = int(math.ceil(warmup_fraction * total_steps))
    if step < w:
        return lr_max * (step + 1) / w
    if step >= total_steps:
        return 0.0
    return lr_max * 0.5 * (1.0 + math.cos(math.pi * (step - w) / (total_steps - w)))
