"""fp64 CPU oracle for the parameter update of the attention-distillation loop (Sec. 3.3, Alg. "distil": the line
phi <- phi - eta grad_phi L; the appendix's training details name AdamW, learning rate 1e-3, for this stage).

TEST INFRASTRUCTURE ONLY.  It shares no code with the GPU library and must never be imported by the product path.

Two rules, both elementwise over a parameter tensor:
  * `sgd_step`: the update exactly as Alg. "distil" prints it, with the factor 1 / (m |T|) of its loss line as
    `grad_scale` (the gradient entry point returns the gradient of the plain sum).
  * `adamw_step`: Adam with decoupled weight decay (Loshchilov & Hutter): the parameter is first shrunk by
    lr * weight_decay, then moved along the bias-corrected first moment over the root of the bias-corrected second
    moment plus eps.  `step` counts from 1.

Pins (tests/test_param_update_oracle.py): torch.optim.SGD and torch.optim.AdamW in float64 over several steps, the
closed form of the first AdamW step (a move of lr * sign(g) when eps and the decay are zero) and planted mistakes.
No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def sgd_step(param, grad, lr: float, grad_scale: float = 1.0):
    """phi - eta * (grad_scale * grad)."""
    return np.asarray(param, dtype=np.float64) - lr * (grad_scale * np.asarray(grad, dtype=np.float64))


def adamw_step(param, grad, m, v, step: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
               weight_decay: float = 0.01, grad_scale: float = 1.0):
    """One AdamW update; returns (param, m, v)."""
    if step < 1:
        raise ValueError("step counts from 1")
    p = np.asarray(param, dtype=np.float64)
    g = grad_scale * np.asarray(grad, dtype=np.float64)
    p = p * (1.0 - lr * weight_decay)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    p = p - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p, m, v
