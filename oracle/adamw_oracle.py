"""Float64 CPU oracle of the AdamW step used for vector-valued parameters (TEST INFRASTRUCTURE ONLY).

Sec. 4.1 (text above Alg. 1): parameters that are not matrices (embeddings, biases, norm gains)
are not orthogonalised; they fall back to AdamW.  The paper gives no formula of its own and cites
the decoupled-weight-decay Adam of Loshchilov and Hutter; that published algorithm, written out:

    m_t = beta1 m_{t-1} + (1 - beta1) g_t
    v_t = beta2 v_{t-1} + (1 - beta2) g_t^2
    mhat = m_t / (1 - beta1^t),   vhat = v_t / (1 - beta2^t)
    w_t = w_{t-1} - eta (mhat / (sqrt(vhat) + eps) + lambda w_{t-1})

with m_0 = v_0 = 0, t counted from 1, the decay acting on the old w and scaled by eta (the same
convention as Eq. muon_update for the matrices).

Imported only by tests, the smoke check and the benchmark's CPU-baseline leg.  Pins
(tests/test_adamw_oracle_pins.py): torch.optim.AdamW on float64 CPU tensors (a library routine
that implements the same published algorithm); the constant-gradient closed form; the first
step, which moves every element by eta g / (|g| + eps) whatever the betas.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class AdamWHParams:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1

    def f32(self) -> "AdamWHParams":
        r = lambda v: float(np.float32(v))
        return AdamWHParams(r(self.lr), r(self.beta1), r(self.beta2), r(self.eps), r(self.weight_decay))


class AdamWOracle:
    """State {m, v, t} and the step for ONE parameter tensor (any shape), float64."""

    def __init__(self, shape):
        self.m = np.zeros(shape, dtype=np.float64)
        self.v = np.zeros(shape, dtype=np.float64)
        self.t = 0

    def step(self, w: np.ndarray, g: np.ndarray, hp: AdamWHParams) -> np.ndarray:
        """Returns w_t (float64); w is not modified."""
        w = np.asarray(w, dtype=np.float64)
        g = np.asarray(g, dtype=np.float64)
        self.t += 1
        self.m = hp.beta1 * self.m + (1.0 - hp.beta1) * g
        self.v = hp.beta2 * self.v + (1.0 - hp.beta2) * g * g
        mhat = self.m / (1.0 - hp.beta1 ** self.t)
        vhat = self.v / (1.0 - hp.beta2 ** self.t)
        return w - hp.lr * (mhat / (np.sqrt(vhat) + hp.eps) + hp.weight_decay * w)
