"""CPU oracle for the optimizer update of a training step -- TEST INFRASTRUCTURE ONLY.

The paper trains with AdamW (Sec. 4, experimental setup) and also reports that
plain SGD behaves alike; it gives no hyper-parameters and no formula, so the
update is the published one (Adam with decoupled weight decay), written out
here in float64, one line per quantity, no fusion:

    m_t   = beta1 * m_{t-1} + (1 - beta1) * g
    v_t   = beta2 * v_{t-1} + (1 - beta2) * g * g
    mhat  = m_t / (1 - beta1**t)
    vhat  = v_t / (1 - beta2**t)
    theta = theta - lr * (mhat / (sqrt(vhat) + eps) + weight_decay * theta)

Readings where the paper is silent: eps is added outside the square root; the
decay term uses the parameter value from before the step; the step counter t
starts at 1; no amsgrad, no gradient clipping.  `sgd_step` is the plain
theta - lr * g.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this module; it shares no code with the HIP path.  Pins
(tests/test_adamw_oracle_pins.py): an independent library implementation run in
float64, the closed form of the first step from zero moments, pure decay under
zero gradients, the constant-gradient fixed point, and scale invariance.  Not
"parity unpinned".
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def adamw_step(theta, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """One AdamW update.  Arrays of one shape; returns (theta, m, v) as new float64 arrays."""
    theta = np.asarray(theta, F64)
    g = np.asarray(g, F64)
    m = np.asarray(m, F64)
    v = np.asarray(v, F64)
    if t < 1:
        raise ValueError("the step counter starts at 1")
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    mhat = m_new / (1.0 - beta1 ** t)
    vhat = v_new / (1.0 - beta2 ** t)
    theta_new = theta - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * theta)
    return theta_new, m_new, v_new


def sgd_step(theta, g, lr):
    return np.asarray(theta, F64) - lr * np.asarray(g, F64)
