"""Per-adapter AdamW step.  Test infrastructure only.

Packed LoRA fine-tuning keeps, for every adapter, its own parameters and its own optimizer state
(paper section 2.4); the memory model of appendix B counts three gradient-sized buffers per adapter
"in the popular AdamW optimizer": the gradient, the momentum and the velocity.  The learning rate
is one of the per-job hyperparameters (Table 1), so every adapter steps with its own.

The paper does not print the update rule; this is AdamW as published (Loshchilov & Hutter,
"Decoupled weight decay regularization"), in the order the common frameworks apply it: decay the
parameter, update the two moments, correct their bias with the adapter's own step count t, step:

    theta <- theta * (1 - lr * wd)
    m     <- beta1 * m + (1 - beta1) * g
    v     <- beta2 * v + (1 - beta2) * g * g
    theta <- theta - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)

All arithmetic in fp64, element by element; nothing is fused or reordered.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np


@dataclass
class Hyper:
    """Hyperparameters of one adapter; ``step`` is t of the update being taken (1 for the first)."""
    lr: float
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    step: int = 1
    grad_scale: float = 1.0   # the adapter's own multiplier on its gradient (see step_tensor)


def step_tensor(theta, g, m, v, hp: Hyper) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One AdamW update of one tensor: returns (theta, m, v) after the step, all fp64.

    Every adapter of a packed run has its own data and its own loss (section 2.4), so what turns the
    gradient the backward pass wrote into the gradient of that adapter's objective - the normalisation
    by its own batch size (a per-job knob, Table 1), a clipping coefficient from its own gradient norm -
    is a factor per adapter: g <- grad_scale * g before the rule is applied."""
    theta = np.asarray(theta, dtype=np.float64)
    g = float(hp.grad_scale) * np.asarray(g, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    lr, b1, b2 = float(hp.lr), float(hp.beta1), float(hp.beta2)
    theta = theta * (1.0 - lr * float(hp.weight_decay))
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    m_hat = m / (1.0 - b1 ** int(hp.step))
    v_hat = v / (1.0 - b2 ** int(hp.step))
    theta = theta - lr * m_hat / (np.sqrt(v_hat) + float(hp.eps))
    return theta, m, v


def step_adapters(A: Sequence, B: Sequence, dA: Sequence, dB: Sequence, mA: Sequence, vA: Sequence,
                  mB: Sequence, vB: Sequence, hp: Sequence[Hyper]):
    """Every adapter's A_k and B_k with that adapter's hyperparameters.

    Returns (A, B, mA, vA, mB, vB) as lists of fp64 arrays."""
    out = [[], [], [], [], [], []]
    for k in range(len(A)):
        a, ma, va = step_tensor(A[k], dA[k], mA[k], vA[k], hp[k])
        b, mb, vb = step_tensor(B[k], dB[k], mB[k], vB[k], hp[k])
        for lst, val in zip(out, (a, b, ma, va, mb, vb)):
            lst.append(val)
    return tuple(out)
