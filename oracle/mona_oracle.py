"""Float64 CPU oracle of the MONA optimizer step (TEST INFRASTRUCTURE ONLY).

This file is the slow, plain reference the HIP path is checked against.  It is
imported only by the tests, the smoke check and the benchmark's CPU-baseline
leg; the product path never routes through it.  It shares no code with the HIP
sources and imports nothing from the package's binding.

Everything follows Algorithm 1 of the paper line by line, one matrix at a
time (Sec. 3.1: the method is defined for a single matrix W of shape m x n),
in numpy float64:

    D_k   = G_k - G_{k-1}                              (Alg. 1, difference line; Eq. alto_diff)
    A_k   = beta_a A_{k-1} + (1 - beta_a) D_k          (Eq. alto_accel)
    Gt_k  = G_k + alpha A_k                            (Eq. alto_grad)
    M_k   = mu M_{k-1} + Gt_k                          (Eq. muon_momentum, fed with Gt_k)
    O_k   = NewtonSchulz(M_k, T)                       (Eq. newton_schulz, X_0 = M_k / ||M_k||_F)
    W_k+1 = W_k - eta (gamma O_k + lambda W_k)         (Eq. muon_update), gamma = 0.2 sqrt(max(m, n))
    G_{k-1} <- G_k                                     (Alg. 1, last line of the loop)

with M_0 = A_0 = G_0 = 0 (Alg. 1, initialisation line).

Readings taken where the paper is silent (each listed in the design notes):
  * the first step uses G_0 = 0 literally, so D_1 = G_1;
  * X_0 = M / (||M||_F + eps) with eps = 0 by default, and X_0 = 0 when the
    denominator is 0 (then O = 0 and only weight decay acts);
  * the Newton-Schulz input is M_k itself, no look-ahead combination;
  * weight decay multiplies the old W_k and is scaled by eta.

Pins (tests/test_oracle_pins.py): alpha = 0 against an independently written
Muon step built on the SVD; constant gradients; EMA / momentum closed forms;
Lemma 1 / Lemma 2 norm bounds; Newton-Schulz against U diag(p^T(sigma)) V^T
from LAPACK's SVD, rank-one and scaled-identity closed forms, transpose
identity, T = 0; update special cases.  End-to-end composition has no
printed numeric example in the paper: "parity unpinned" beyond those pins.

MONA-Lite (Sec. 6.3, low-precision state): `state_dtype="bf16"` rounds the
stored G_{k-1} and A_k to bfloat16 (round-to-nearest-even) after each step's
arithmetic, the arithmetic itself unchanged: G~_k and M_k use the unrounded
A_k of the same step, the next step's D and EMA read the rounded values back,
and M stays full precision.  The paper prints no numbers for this variant;
the reading is fixed by a two-step example worked by hand in exact fractions
(tests/golden/bf16_state_worked_example.txt), which a rounding placed
anywhere else fails.

One-buffer form of the acceleration term (`accel_form="one_buffer"`; the
goal of Sec. 6.3's streaming variant, no stored G_{k-1}, reached by algebra
instead of by aliasing the gradient slot).  Substituting D_k in Eq.
alto_accel gives A_k = [beta_a A_{k-1} - (1 - beta_a) G_{k-1}] + (1 - beta_a) G_k,
so carrying the bracket C_k is enough:

    A_k     = C_k + (1 - beta_a) G_k,        C_1 = 0   (A_0 = G_0 = 0)
    C_{k+1} = beta_a A_k - (1 - beta_a) G_k

In exact arithmetic this IS Alg. 1 (pinned: both forms agree to 1e-12 in
float64, and C_{k+1} = -(1 - beta_a)^2 sum_j beta_a^{k-j} G_j in closed form);
the separate code path exists only to say where the bf16 rounding falls when
the single buffer is stored in bfloat16 (on C, after each step).  beta_a must
not change between steps in this form.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

# Newton-Schulz coefficients printed under Eq. newton_schulz
NS_A, NS_B, NS_C = 3.4445, -4.7750, 2.0315


@dataclass
class OracleHParams:
    """Alg. 1 REQUIRE line.  Values are stored as given; callers that compare
    against an fp32 ABI pass the float32-rounded values (see `f32`)."""
    lr: float = 2e-2
    momentum: float = 0.95
    beta_a: float = 0.9
    alpha: float = -5.0
    weight_decay: float = 0.1
    ns_steps: int = 5
    ns_a: float = NS_A
    ns_b: float = NS_B
    ns_c: float = NS_C
    ns_eps: float = 0.0
    gamma_coeff: float = 0.2

    def f32(self) -> "OracleHParams":
        """The same hyper-parameters after a round trip through float32, i.e.
        the exact real numbers a float32 ABI carries."""
        r = lambda v: float(np.float32(v))
        return OracleHParams(r(self.lr), r(self.momentum), r(self.beta_a), r(self.alpha),
                             r(self.weight_decay), int(self.ns_steps), r(self.ns_a),
                             r(self.ns_b), r(self.ns_c), r(self.ns_eps), r(self.gamma_coeff))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (ties to even), returned as
    float64.  bfloat16 = the top 16 bits of an IEEE float32."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = rounded.astype(np.uint32).view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if nan.any():
        out = np.where(nan, np.nan, out)
    return out


def newton_schulz(M: np.ndarray, steps: int = 5, a: float = NS_A, b: float = NS_B,
                  c: float = NS_C, eps: float = 0.0) -> np.ndarray:
    """Eq. newton_schulz, literal form for any shape:
    X_0 = M / (||M||_F + eps);  X_{t+1} = a X_t + b (X_t X_t^T) X_t + c (X_t X_t^T)^2 X_t."""
    M = np.asarray(M, dtype=np.float64)
    den = np.sqrt(np.sum(M * M)) + eps
    if den == 0.0:
        X = np.zeros_like(M)
    else:
        X = M / den
    for _ in range(int(steps)):
        S = X @ X.T
        X = a * X + b * (S @ X) + c * (S @ (S @ X))
    return X


def newton_schulz_short_side(M: np.ndarray, steps: int = 5, a: float = NS_A, b: float = NS_B,
                             c: float = NS_C, eps: float = 0.0) -> np.ndarray:
    """The same iteration with the Gram matrix taken on the short side: for a
    tall X, (X X^T) X = X (X^T X), so X_{t+1} = X (a I + b S + c S^2), S = X^T X.
    Only used to pin that identity; the oracle proper uses `newton_schulz`."""
    M = np.asarray(M, dtype=np.float64)
    m, n = M.shape
    if m <= n:
        return newton_schulz(M, steps, a, b, c, eps)
    den = np.sqrt(np.sum(M * M)) + eps
    X = np.zeros_like(M) if den == 0.0 else M / den
    for _ in range(int(steps)):
        S = X.T @ X
        X = a * X + X @ (b * S + c * (S @ S))
    return X


def update_scale(m: int, n: int, gamma_coeff: float = 0.2) -> float:
    """gamma = 0.2 sqrt(max(m, n))  (scaling-factor equation after Eq. newton_schulz)."""
    return gamma_coeff * float(np.sqrt(float(max(m, n))))


class MonaOracle:
    """State {G_{k-1}, A, M} and the step of Alg. 1 for ONE matrix, float64."""

    def __init__(self, shape, state_dtype: str = "f32", accel_form: str = "two_buffer"):
        m, n = shape
        self.shape = (int(m), int(n))
        self.G_prev = np.zeros(self.shape, dtype=np.float64)
        self.A = np.zeros(self.shape, dtype=np.float64)
        self.M = np.zeros(self.shape, dtype=np.float64)
        self.C = np.zeros(self.shape, dtype=np.float64)   # one-buffer form only
        self.k = 0
        assert state_dtype in ("f32", "bf16")
        assert accel_form in ("two_buffer", "one_buffer")
        self.state_dtype = state_dtype
        self.accel_form = accel_form
        # results of the last step, kept for inspection
        self.norm = 0.0
        self.O: Optional[np.ndarray] = None
        self.G_tilde: Optional[np.ndarray] = None

    def elementwise(self, G: np.ndarray, hp: OracleHParams) -> np.ndarray:
        """Difference, acceleration EMA, accelerated gradient, momentum and the
        state roll; returns M_k."""
        G = np.asarray(G, dtype=np.float64)
        assert G.shape == self.shape
        if self.accel_form == "one_buffer":
            # A_k from the carried bracket; self.A and self.G_prev are kept for inspection only
            self.A = self.C + (1.0 - hp.beta_a) * G
            self.G_tilde = G + hp.alpha * self.A
            self.M = hp.momentum * self.M + self.G_tilde
            self.C = hp.beta_a * self.A - (1.0 - hp.beta_a) * G
            if self.state_dtype == "bf16":
                self.C = round_to_bf16(self.C)
            self.G_prev = G.copy()
            self.k += 1
            return self.M
        D = G - self.G_prev
        self.A = hp.beta_a * self.A + (1.0 - hp.beta_a) * D
        self.G_tilde = G + hp.alpha * self.A
        self.M = hp.momentum * self.M + self.G_tilde
        self.G_prev = G.copy()
        if self.state_dtype == "bf16":
            self.A = round_to_bf16(self.A)
            self.G_prev = round_to_bf16(self.G_prev)
        self.k += 1
        return self.M

    def step(self, W: np.ndarray, G: np.ndarray, hp: OracleHParams) -> np.ndarray:
        """One full step; returns W_{k+1} (float64).  W is not modified."""
        W = np.asarray(W, dtype=np.float64)
        assert W.shape == self.shape
        M = self.elementwise(G, hp)
        self.norm = float(np.sqrt(np.sum(M * M)))
        self.O = newton_schulz(M, hp.ns_steps, hp.ns_a, hp.ns_b, hp.ns_c, hp.ns_eps)
        gamma = update_scale(self.shape[0], self.shape[1], hp.gamma_coeff)
        return W - hp.lr * (gamma * self.O + hp.weight_decay * W)


def run_oracle(weights, grads_per_step, hp: OracleHParams, state_dtype: str = "f32",
               round_w_to_bf16=None):
    """Run K steps over a list of matrices.

    weights: list of arrays (initial W, any float dtype; widened exactly).
    grads_per_step: grads_per_step[k][i] = gradient of matrix i at step k.
    round_w_to_bf16: optional list of bools; where True the parameter is stored
      in bfloat16, i.e. W_{k+1} is rounded after every step (the stored
      parameter dtype is the caller's choice, not part of Alg. 1).
    Returns (oracles, W_final list, history) where history[k][i] holds copies
    of (G_prev, A, M, norm, O, W) after step k.
    """
    oracles = [MonaOracle(np.asarray(w).shape, state_dtype) for w in weights]
    Ws = [np.asarray(w, dtype=np.float64).copy() for w in weights]
    history = []
    for grads in grads_per_step:
        snap = []
        for i, (orc, g) in enumerate(zip(oracles, grads)):
            Wn = orc.step(Ws[i], np.asarray(g, dtype=np.float64), hp)
            if round_w_to_bf16 is not None and round_w_to_bf16[i]:
                Wn = round_to_bf16(Wn)
            Ws[i] = Wn
            snap.append(dict(G_prev=orc.G_prev.copy(), A=orc.A.copy(), M=orc.M.copy(),
                             norm=orc.norm, O=orc.O.copy(), W=Wn.copy()))
        history.append(snap)
    return oracles, Ws, history
