"""CPU oracle of the parameter update that closes a training iteration (TEST INFRASTRUCTURE ONLY).

This file is test infrastructure: only tests, the smoke check and the bench's cpu_baseline leg
may import it.  It shares no code with the HIP library.

The training pipeline of Section 2.1 ends with an update of the parameters from the gradients,
and Section 3.1 counts the optimizer's state among the memory that does not depend on the input
size.  The paper names no optimizer; the update used here is Adam with decoupled weight decay
(AdamW, Loshchilov and Hutter 2019, Algorithm 2), written out element by element in fp64:

    m_t = b1 m_{t-1} + (1 - b1) g
    v_t = b2 v_{t-1} + (1 - b2) g^2
    p_t = p_{t-1} - lr * ( (m_t / (1 - b1^t)) / (sqrt(v_t / (1 - b2^t)) + eps) + wd * p_{t-1} )

Reading where the paper is silent: weight decay applies to tensors with two or more dimensions
(weight matrices and embedding tables), not to biases and LayerNorm scales / shifts.  With a
bf16 model the update runs on fp32 master copies and the bf16 parameter is the master rounded to
nearest-even; the oracle mirrors only that rounding (`quantise`), everything else stays fp64.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, Optional

import numpy as np


@dataclass
class AdamW:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    t: int = 0
    m: Dict[str, np.ndarray] = field(default_factory=dict)
    v: Dict[str, np.ndarray] = field(default_factory=dict)

    def step(self, params: Dict[str, np.ndarray], grads: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
        """One update of every tensor; returns the new parameters (fp64), inputs untouched."""
        self.t += 1
        c1 = 1.0 - self.beta1 ** self.t
        c2 = 1.0 - self.beta2 ** self.t
        out = {}
        for k, p in params.items():
            p = np.asarray(p, dtype=np.float64)
            g = np.asarray(grads[k], dtype=np.float64)
            m = self.m.get(k, np.zeros_like(p))
            v = self.v.get(k, np.zeros_like(p))
            m = self.beta1 * m + (1.0 - self.beta1) * g
            v = self.beta2 * v + (1.0 - self.beta2) * g * g
            self.m[k], self.v[k] = m, v
            wd = self.weight_decay if p.ndim >= 2 else 0.0
            out[k] = p - self.lr * ((m / c1) / (np.sqrt(v / c2) + self.eps) + wd * p)
        return out
