"""Pins for the float64 oracle: every check here compares the oracle with
something other than itself -- closed forms, LAPACK's SVD, the constants the
paper prints, invariants from its lemmas, special cases that reduce to plain
Muon -- so that a dropped term, a wrong sign or a transposed operand in
oracle/mona_oracle.py fails at least one of them (see the planted-mistake
tests at the end).  CPU only.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import mona_oracle as orc
from oracle.mona_oracle import MonaOracle, OracleHParams, newton_schulz_short_side


def newton_schulz(*args, **kwargs):
    # looked up at call time so that the planted-mistake test can swap it
    return orc.newton_schulz(*args, **kwargs)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def read_golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = (s.strip() for s in line.split("=", 1))
            out[k] = float(v)
    return out


def scalar_poly(s, a, b, c):
    """p(s) = a s + b s^3 + c s^5: what one Newton-Schulz iteration does to a
    singular value (Eq. newton_schulz applied to X = U diag(s) V^T)."""
    return s * (a + s * s * (b + c * s * s))


def scalar_poly_iter(s, T, a, b, c):
    for _ in range(T):
        s = scalar_poly(s, a, b, c)
    return s


def rng(seed):
    return np.random.default_rng(seed)


def grad_stream(shape, seed, steps, sigma=1e-3, rho=0.9):
    r = rng(seed)
    out, prev = [], None
    for _ in range(steps):
        z = r.standard_normal(shape)
        g = sigma * z if prev is None else rho * prev + math.sqrt(1 - rho * rho) * sigma * z
        out.append(g)
        prev = g
    return out


# ----------------------------------------------------------------------------
# constants the paper prints
# ----------------------------------------------------------------------------
def test_defaults_match_printed_constants():
    g = read_golden()
    hp = OracleHParams()
    assert (hp.ns_a, hp.ns_b, hp.ns_c) == (g["ns_a"], g["ns_b"], g["ns_c"])
    assert hp.ns_steps == int(g["ns_steps"])
    assert hp.gamma_coeff == g["gamma_coeff"]
    # the hyper-parameter rule of the Limitations section reproduces the printed pairs
    for i in (1, 2, 3):
        beta = g[f"rule_beta_a_{i}"]
        assert -1.0 / (2.0 * (1.0 - beta)) == pytest.approx(g[f"rule_alpha_{i}"], rel=1e-12)
    # default benchmark pair follows the same rule
    assert -1.0 / (2.0 * (1.0 - hp.beta_a)) == pytest.approx(hp.alpha, rel=1e-12)


def test_update_scale_formula():
    assert orc.update_scale(256, 512) == pytest.approx(0.2 * math.sqrt(512), rel=1e-15)
    assert orc.update_scale(8192, 2048) == pytest.approx(0.2 * math.sqrt(8192), rel=1e-15)
    assert orc.update_scale(7, 7) == pytest.approx(0.2 * math.sqrt(7), rel=1e-15)


# ----------------------------------------------------------------------------
# bf16 rounding helper against torch's conversion (a library routine)
# ----------------------------------------------------------------------------
def test_round_to_bf16_matches_torch():
    r = rng(5)
    x = np.concatenate([
        r.standard_normal(4096) * 10.0 ** r.integers(-20, 20, 4096),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, 3.0e38, -3.0e38,
                  1e-40, float("inf"), -float("inf")]),
    ])
    x32 = x.astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_to_bf16(x32.astype(np.float64))
    assert np.array_equal(got, want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert orc.round_to_bf16(np.array([1.00390625]))[0] == 1.0
    assert orc.round_to_bf16(np.array([1.01171875]))[0] == 1.015625


# ----------------------------------------------------------------------------
# (4) EMA and momentum recurrences against their closed forms
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("beta_a,alpha,mu", [(0.9, -5.0, 0.95), (0.98, -25.0, 0.9), (0.5, 0.7, 0.0)])
def test_ema_and_momentum_closed_forms(beta_a, alpha, mu):
    shape, K = (7, 11), 9
    G = grad_stream(shape, 11, K)
    hp = OracleHParams(beta_a=beta_a, alpha=alpha, momentum=mu)
    o = MonaOracle(shape)
    Gt_hist = []
    for k in range(1, K + 1):
        o.elementwise(G[k - 1], hp)
        Gt_hist.append(o.G_tilde.copy())
        # A_k = (1 - beta) sum_j beta^(k-j) (G_j - G_{j-1}),  G_0 = 0
        A_cf = np.zeros(shape)
        for j in range(1, k + 1):
            Gjm1 = G[j - 2] if j >= 2 else np.zeros(shape)
            A_cf += (1 - beta_a) * beta_a ** (k - j) * (G[j - 1] - Gjm1)
        # equivalent summation-by-parts form
        A_cf2 = G[k - 1].copy()
        for j in range(1, k):
            A_cf2 -= (1 - beta_a) * beta_a ** (k - 1 - j) * G[j - 1]
        A_cf2 *= (1 - beta_a)
        np.testing.assert_allclose(o.A, A_cf, rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(o.A, A_cf2, rtol=1e-11, atol=1e-18)
        np.testing.assert_allclose(o.G_tilde, G[k - 1] + alpha * A_cf, rtol=1e-12, atol=1e-18)
        M_cf = sum(mu ** (k - j) * Gt_hist[j - 1] for j in range(1, k + 1))
        np.testing.assert_allclose(o.M, M_cf, rtol=1e-12, atol=1e-18)
        assert np.array_equal(o.G_prev, G[k - 1])
    assert o.k == K


def test_first_step_with_the_rule_halves_the_gradient():
    # alpha (1 - beta_a) = -1/2 exactly  =>  Gt_1 = G_1 / 2 and M_1 = G_1 / 2
    hp = OracleHParams(beta_a=0.75, alpha=-2.0, momentum=0.95)
    G = grad_stream((5, 6), 3, 1)[0]
    o = MonaOracle((5, 6))
    o.elementwise(G, hp)
    assert np.array_equal(o.A, 0.25 * G)
    assert np.array_equal(o.G_tilde, 0.5 * G)
    assert np.array_equal(o.M, 0.5 * G)


# ----------------------------------------------------------------------------
# (2) constant gradients
# ----------------------------------------------------------------------------
def test_constant_gradient_pure_decay_and_zero_acceleration():
    shape = (6, 4)
    g = rng(2).standard_normal(shape) * 1e-3
    hp = OracleHParams(beta_a=0.9, alpha=-5.0)
    # (2a) Alg. 1 literally (G_0 = 0): after step 1 the difference is exactly 0
    # and A only decays: A_k = beta^(k-1) (1 - beta) g
    o = MonaOracle(shape)
    o.elementwise(g, hp)
    A1 = o.A.copy()
    np.testing.assert_allclose(A1, (1 - 0.9) * g, rtol=1e-15)
    for k in range(2, 8):
        prev = o.A.copy()
        o.elementwise(g, hp)
        assert np.array_equal(o.A, hp.beta_a * prev)
        np.testing.assert_allclose(o.A, 0.9 ** (k - 1) * 0.1 * g, rtol=1e-13)
    # (2b) previous-gradient buffer already holding g: acceleration is exactly 0
    # at every step and the momentum is plain Muon's geometric sum
    o = MonaOracle(shape)
    o.G_prev = g.copy()
    M_ref = np.zeros(shape)
    for k in range(1, 8):
        o.elementwise(g, hp)
        M_ref = hp.momentum * M_ref + g
        assert not o.A.any()
        assert np.array_equal(o.G_tilde, g)
        assert np.array_equal(o.M, M_ref)


# ----------------------------------------------------------------------------
# Lemma 1 / Lemma 2 norm bounds
# ----------------------------------------------------------------------------
def test_lemma_norm_bounds():
    shape, K = (16, 24), 40
    G = grad_stream(shape, 21, K)
    Gmax = max(np.linalg.norm(g) for g in G)
    hp = OracleHParams(beta_a=0.9, alpha=-5.0, momentum=0.95)
    o = MonaOracle(shape)
    for k in range(1, K + 1):
        o.elementwise(G[k - 1], hp)
        assert np.linalg.norm(o.A) <= 2 * Gmax * (1 - hp.beta_a ** k) * (1 + 1e-12)
        assert np.linalg.norm(o.G_tilde) <= Gmax * (1 + 2 * abs(hp.alpha)) * (1 + 1e-12)
        assert np.linalg.norm(o.M) <= Gmax * (1 + 2 * abs(hp.alpha)) / (1 - hp.momentum) * (1 + 1e-12)


# ----------------------------------------------------------------------------
# (3) Newton-Schulz against the SVD
# ----------------------------------------------------------------------------
def ns_via_svd(M, T, a, b, c, eps=0.0):
    """X_T = U diag(p^T(sigma_i / ||M||_F)) V^T: the polynomial is odd, so it
    acts on the singular values only."""
    U, s, Vt = np.linalg.svd(M, full_matrices=False)
    den = math.sqrt(float(np.sum(s * s))) + eps
    s0 = s / den
    sT = np.array([scalar_poly_iter(x, T, a, b, c) for x in s0])
    return (U * sT) @ Vt, s0, sT


@pytest.mark.parametrize("shape", [(8, 8), (12, 30), (30, 12), (1, 9), (9, 1), (64, 96)])
@pytest.mark.parametrize("T", [0, 1, 2, 5])
def test_newton_schulz_matches_svd_closed_form(shape, T):
    M = rng(100 + shape[0] * 7 + shape[1]).standard_normal(shape) * 1e-3
    want, _, _ = ns_via_svd(M, T, orc.NS_A, orc.NS_B, orc.NS_C)
    got = newton_schulz(M, T)
    assert np.linalg.norm(got - want) <= 1e-10 * max(np.linalg.norm(want), 1e-300)


def test_newton_schulz_T0_is_frobenius_normalisation():
    M = rng(4).standard_normal((5, 9))
    np.testing.assert_allclose(newton_schulz(M, 0), M / np.linalg.norm(M), rtol=1e-15)
    assert np.linalg.norm(newton_schulz(M, 0)) == pytest.approx(1.0, rel=1e-15)
    assert not newton_schulz(np.zeros((3, 4)), 5).any()          # zero matrix stays zero
    # eps enters the denominator only
    np.testing.assert_allclose(newton_schulz(M, 0, eps=0.5), M / (np.linalg.norm(M) + 0.5), rtol=1e-15)


def test_newton_schulz_polar_factor_and_singular_value_band():
    a, b, c = orc.NS_A, orc.NS_B, orc.NS_C
    # the quintic's interior extrema on (0, 1.3): roots of p'(s) = a + 3 b s^2 + 5 c s^4
    disc = math.sqrt(9 * b * b - 20 * a * c)
    s_max = math.sqrt((-3 * b - disc) / (10 * c))
    s_min = math.sqrt((-3 * b + disc) / (10 * c))
    hi, lo = scalar_poly(s_max, a, b, c), scalar_poly(s_min, a, b, c)
    assert s_max == pytest.approx(0.55453, abs=1e-4) and hi == pytest.approx(1.20237, abs=1e-4)
    assert s_min == pytest.approx(1.05014, abs=1e-4) and lo == pytest.approx(0.68183, abs=1e-4)
    # [lo, hi] is mapped into itself, so once a singular value is inside it stays inside
    grid = np.linspace(lo, hi, 20001)
    img = scalar_poly(grid, a, b, c)
    assert img.min() >= lo - 1e-12 and img.max() <= hi + 1e-12
    # a well-conditioned tiny matrix: all sigma_i / ||M||_F >= 0.05 => 5 iterations land in the band
    r = rng(8)
    U, _ = np.linalg.qr(r.standard_normal((6, 6)))
    V, _ = np.linalg.qr(r.standard_normal((10, 6)))
    s = np.array([1.0, 0.8, 0.6, 0.5, 0.35, 0.25])
    M = (U * s) @ V.T
    O = newton_schulz(M, 5)
    sv = np.linalg.svd(O, compute_uv=False)
    assert sv.min() >= lo - 1e-9 and sv.max() <= hi + 1e-9
    # distance to the polar factor U V^T is what the band implies, not more
    polar = U @ V.T
    assert np.linalg.norm(O - polar, 2) <= max(hi - 1, 1 - lo) + 1e-9
    # O has the same singular vectors as M: U^T O V is diagonal
    core = U.T @ O @ V
    assert np.linalg.norm(core - np.diag(np.diag(core))) <= 1e-10
    # tiny singular values are amplified by about a per step: p^T(s) ~ a^T s
    tiny = 1e-9
    assert scalar_poly_iter(tiny, 5, a, b, c) == pytest.approx(a ** 5 * tiny, rel=1e-6)


def test_newton_schulz_rank_one_and_scaled_identity():
    a, b, c = orc.NS_A, orc.NS_B, orc.NS_C
    r = rng(12)
    u, v = r.standard_normal(9), r.standard_normal(14)
    M = 3.7e-3 * np.outer(u, v)
    want = scalar_poly_iter(1.0, 5, a, b, c) * np.outer(u / np.linalg.norm(u), v / np.linalg.norm(v))
    np.testing.assert_allclose(newton_schulz(M, 5), want, rtol=1e-9, atol=1e-12)
    assert scalar_poly_iter(1.0, 5, a, b, c) == pytest.approx(0.6964364094697522, rel=1e-12)
    # M = kappa [I_p 0]: every singular value is 1/sqrt(p) after normalisation
    for p, q in [(4, 4), (16, 40), (256, 300)]:
        M = np.zeros((p, q))
        M[:, :p] = -2.5 * np.eye(p)
        O = newton_schulz(M, 5)
        val = scalar_poly_iter(1.0 / math.sqrt(p), 5, a, b, c)
        ref = np.zeros((p, q))
        ref[:, :p] = -val * np.eye(p)
        np.testing.assert_allclose(O, ref, rtol=0, atol=1e-11)
    assert scalar_poly_iter(1 / 16.0, 5, a, b, c) == pytest.approx(1.070524447724669, rel=1e-12)
    # the short sides of the benchmark shapes: p^5(1 / sqrt(p)) for p = 1024 and p = 4096, and the oracle
    # itself on kappa [I_p 0] at p = 1024 (one 1024 x 1024 Gram matrix per iteration: well under a second)
    assert scalar_poly_iter(1 / 32.0, 5, a, b, c) == pytest.approx(1.1329236117054717, rel=1e-12)
    assert scalar_poly_iter(1 / 64.0, 5, a, b, c) == pytest.approx(0.9025257529666177, rel=1e-12)
    M = np.zeros((1024, 1056))
    M[:, :1024] = 0.75 * np.eye(1024)
    O = newton_schulz(M, 5)
    ref = np.zeros_like(M)
    ref[:, :1024] = 1.1329236117054717 * np.eye(1024)
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-11)


@pytest.mark.parametrize("shape", [(40, 12), (12, 40), (25, 25), (33, 1)])
def test_newton_schulz_transpose_and_short_side_identities(shape):
    M = rng(31 + shape[0]).standard_normal(shape) * 2e-3
    X = newton_schulz(M, 5)
    Xt = newton_schulz(M.T, 5)
    assert np.linalg.norm(X - Xt.T) <= 1e-12 * np.linalg.norm(X)
    Xs = newton_schulz_short_side(M, 5)
    assert np.linalg.norm(X - Xs) <= 1e-12 * np.linalg.norm(X)


# ----------------------------------------------------------------------------
# (1) alpha = 0 is plain Muon, written independently on top of the SVD
# ----------------------------------------------------------------------------
def muon_reference_step(W, M_prev, G, lr, mu, wd, T, a, b, c):
    """Eqs. muon_momentum / muon_ns / muon_update with the orthogonalisation
    evaluated through the SVD instead of matrix iterations."""
    M = mu * M_prev + G
    O, _, _ = ns_via_svd(M, T, a, b, c)
    gamma = 0.2 * math.sqrt(max(W.shape))
    return W - lr * (gamma * O + wd * W), M


@pytest.mark.parametrize("shape", [(16, 24), (24, 16)])
def test_alpha_zero_is_plain_muon(shape):
    K = 4
    G = grad_stream(shape, 77, K)
    W0 = rng(78).standard_normal(shape) * 0.02
    hp = OracleHParams(alpha=0.0, beta_a=0.9)
    o = MonaOracle(shape)
    W, Wm, Mm = W0.copy(), W0.copy(), np.zeros(shape)
    for k in range(K):
        W = o.step(W, G[k], hp)
        Wm, Mm = muon_reference_step(Wm, Mm, G[k], hp.lr, hp.momentum, hp.weight_decay,
                                     hp.ns_steps, hp.ns_a, hp.ns_b, hp.ns_c)
        assert np.array_equal(o.G_tilde, G[k])            # alpha = 0: bitwise the raw gradient
        assert np.array_equal(o.M, Mm)                    # hence bitwise Muon's momentum
        assert np.linalg.norm(W - Wm) <= 1e-10 * np.linalg.norm(Wm)
    assert o.A.any()  # the buffer is still maintained, it just is not used


# ----------------------------------------------------------------------------
# update line special cases
# ----------------------------------------------------------------------------
def test_update_special_cases():
    shape = (6, 10)
    W0 = rng(9).standard_normal(shape) * 0.02
    # zero gradient from a zero state: O = 0, only decoupled weight decay acts
    hp = OracleHParams(lr=0.02, weight_decay=0.1)
    o = MonaOracle(shape)
    W1 = o.step(W0, np.zeros(shape), hp)
    np.testing.assert_allclose(W1, (1 - 0.02 * 0.1) * W0, rtol=1e-15)
    assert not o.O.any() and o.norm == 0.0
    # lambda = 0: Delta W = -eta gamma O
    hp = OracleHParams(lr=0.02, weight_decay=0.0)
    o = MonaOracle(shape)
    G = grad_stream(shape, 10, 1)[0]
    W1 = o.step(W0, G, hp)
    np.testing.assert_allclose(W1 - W0, -0.02 * 0.2 * math.sqrt(10) * o.O, rtol=1e-9, atol=1e-15)
    # the decay multiplies the OLD weights and is scaled by eta
    hp = OracleHParams(lr=0.02, weight_decay=0.1)
    o = MonaOracle(shape)
    W1 = o.step(W0, G, hp)
    np.testing.assert_allclose(W1, (1 - 0.002) * W0 - 0.02 * 0.2 * math.sqrt(10) * o.O, rtol=1e-12, atol=1e-15)
    # RMS sanity for a well-conditioned square case: singular values near 1 give rms(gamma O) ~ 0.2
    n = 64
    Q1, _ = np.linalg.qr(rng(1).standard_normal((n, n)))
    Q2, _ = np.linalg.qr(rng(2).standard_normal((n, n)))
    O = newton_schulz(Q1 @ Q2.T, 5)
    rms = math.sqrt(np.mean((orc.update_scale(n, n) * O) ** 2))
    assert 0.2 * 0.68 <= rms <= 0.2 * 1.21


def test_full_step_composes_the_parts():
    # the composed step equals the parts applied in Alg. 1's order, each part
    # evaluated through its independent form (closed-form EMA, SVD polynomial)
    shape, K = (10, 14), 3
    G = grad_stream(shape, 55, K)
    W = rng(56).standard_normal(shape) * 0.02
    hp = OracleHParams()
    o = MonaOracle(shape)
    Mref = np.zeros(shape)
    for k in range(1, K + 1):
        Wn = o.step(W, G[k - 1], hp)
        A_cf = np.zeros(shape)
        for j in range(1, k + 1):
            Gjm1 = G[j - 2] if j >= 2 else np.zeros(shape)
            A_cf += (1 - hp.beta_a) * hp.beta_a ** (k - j) * (G[j - 1] - Gjm1)
        Mref = hp.momentum * Mref + G[k - 1] + hp.alpha * A_cf
        O_ref, _, _ = ns_via_svd(Mref, hp.ns_steps, hp.ns_a, hp.ns_b, hp.ns_c)
        W_ref = W - hp.lr * (0.2 * math.sqrt(14) * O_ref + hp.weight_decay * W)
        assert np.linalg.norm(Wn - W_ref) <= 1e-9 * np.linalg.norm(W_ref)
        assert o.norm == pytest.approx(np.linalg.norm(Mref), rel=1e-12)
        W = Wn


def test_run_oracle_history_and_bf16_state_variant():
    shapes = [(8, 12), (12, 8)]
    K = 3
    grads = [[grad_stream(s, 60 + i, K)[k] for i, s in enumerate(shapes)] for k in range(K)]
    weights = [rng(70 + i).standard_normal(s) * 0.02 for i, s in enumerate(shapes)]
    hp = OracleHParams()
    _, Wf, hist = orc.run_oracle(weights, grads, hp)
    assert len(hist) == K and len(hist[0]) == 2
    o = MonaOracle(shapes[1])
    W = weights[1]
    for k in range(K):
        W = o.step(W, grads[k][1], hp)
    assert np.array_equal(W, Wf[1]) and np.array_equal(o.M, hist[-1][1]["M"])
    # low-precision state variant: stored G_prev and A are bf16 values, the
    # trajectory stays within bf16 resolution of the full-precision one
    _, Wl, hist_l = orc.run_oracle(weights, grads, hp, state_dtype="bf16")
    for name in ("G_prev", "A"):
        x = hist_l[-1][0][name]
        assert np.array_equal(x, orc.round_to_bf16(x))
    relA = np.abs(hist_l[-1][0]["A"] - hist[-1][0]["A"]).max() / np.abs(hist[-1][0]["A"]).max()
    assert 0 < relA < 3e-2
    # bf16-stored parameters: every stored W is a bf16 value
    _, Wb, _ = orc.run_oracle(weights, grads, hp, round_w_to_bf16=[True, False])
    assert np.array_equal(Wb[0], orc.round_to_bf16(Wb[0]))
    assert np.array_equal(Wb[1], Wf[1])


def test_bf16_state_worked_example():
    """Where the bf16 rounding of the MONA-Lite state falls (Sec. 6.3): a two-step example worked by
    hand in exact fractions, stored under tests/golden with its derivation."""
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "bf16_state_worked_example.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].split()
            if line:
                rows.append([int(x) for x in line])
    assert len(rows) == 4
    hp = OracleHParams(beta_a=0.5, alpha=1.0, momentum=0.5)
    o = MonaOracle((1, 2), state_dtype="bf16")
    for step in (1, 2):
        r = sorted((x for x in rows if x[0] == step), key=lambda x: x[1])
        frac = lambda i: np.array([[r[0][i] / r[0][i + 1], r[1][i] / r[1][i + 1]]])   # dyadic: exact in float64
        M = o.elementwise(frac(2), hp)
        assert np.array_equal(M, frac(4)), (step, M)
        assert np.array_equal(o.G_tilde, frac(6)), (step, o.G_tilde)
        assert np.array_equal(o.A, frac(8)), (step, o.A)
        assert np.array_equal(o.G_prev, frac(10)), (step, o.G_prev)


# ----------------------------------------------------------------------------
# one-buffer form of the acceleration term: same A_k, G~_k, M_k as Alg. 1
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("beta_a,alpha,mu", [(0.9, -5.0, 0.95), (0.975, -20.0, 0.9), (0.3, 1.5, 0.5)])
def test_one_buffer_form_equals_algorithm_one(beta_a, alpha, mu):
    shape, K = (6, 9), 12
    G = grad_stream(shape, 21, K)
    hp = OracleHParams(beta_a=beta_a, alpha=alpha, momentum=mu)
    two, one = MonaOracle(shape), MonaOracle(shape, accel_form="one_buffer")
    for k in range(1, K + 1):
        two.elementwise(G[k - 1], hp)
        one.elementwise(G[k - 1], hp)
        # against the closed form of A_k (itself pinned above), not only against the other code path
        A_cf = np.zeros(shape)
        for j in range(1, k + 1):
            Gjm1 = G[j - 2] if j >= 2 else np.zeros(shape)
            A_cf += (1 - beta_a) * beta_a ** (k - j) * (G[j - 1] - Gjm1)
        np.testing.assert_allclose(one.A, A_cf, rtol=1e-11, atol=1e-17)
        np.testing.assert_allclose(one.A, two.A, rtol=1e-11, atol=1e-17)
        np.testing.assert_allclose(one.G_tilde, two.G_tilde, rtol=1e-11, atol=1e-17)
        np.testing.assert_allclose(one.M, two.M, rtol=1e-11, atol=1e-17)
        # carried bracket in closed form: C_{k+1} = -(1 - beta)^2 sum_{j<=k} beta^(k-j) G_j
        C_cf = -(1 - beta_a) ** 2 * sum(beta_a ** (k - j) * G[j - 1] for j in range(1, k + 1))
        np.testing.assert_allclose(one.C, C_cf, rtol=1e-11, atol=1e-17)
    # a constant gradient from the start with C_1 = -(1 - beta) g (the "G_0 := G_1" start): A_k = 0
    g = G[0]
    o = MonaOracle(shape, accel_form="one_buffer")
    o.C = -(1 - beta_a) * g
    for _ in range(4):
        o.elementwise(g, hp)
        assert np.abs(o.A).max() <= 1e-16 * np.abs(g).max()
    # bf16 storage rounds the carried bracket and nothing else
    ob = MonaOracle(shape, state_dtype="bf16", accel_form="one_buffer")
    for k in range(3):
        ob.elementwise(G[k], hp)
        assert np.array_equal(ob.C, orc.round_to_bf16(ob.C))
    rel = np.abs(ob.M - MonaOracle_run(shape, G[:3], hp).M).max() / np.abs(ob.M).max()
    assert 0 < rel < 3e-2


def MonaOracle_run(shape, grads, hp):
    o = MonaOracle(shape)
    for g in grads:
        o.elementwise(g, hp)
    return o


# ----------------------------------------------------------------------------
# planted mistakes: each plausible slip in the oracle must trip a pin above
# ----------------------------------------------------------------------------
def _pins_pass():
    try:
        test_one_buffer_form_equals_algorithm_one(0.9, -5.0, 0.95)
        test_ema_and_momentum_closed_forms(0.9, -5.0, 0.95)
        test_constant_gradient_pure_decay_and_zero_acceleration()
        test_newton_schulz_matches_svd_closed_form((12, 30), 5)
        test_newton_schulz_matches_svd_closed_form((30, 12), 2)
        test_newton_schulz_rank_one_and_scaled_identity()
        test_update_special_cases()
        test_full_step_composes_the_parts()
        test_alpha_zero_is_plain_muon((16, 24))
        test_bf16_state_worked_example()
    except AssertionError:
        return False
    return True


def test_planted_mistakes_are_caught(monkeypatch):
    assert _pins_pass()

    real_ns = orc.newton_schulz
    real_elem = MonaOracle.elementwise
    real_scale = orc.update_scale

    def ns_dropped_quintic(M, steps=5, a=orc.NS_A, b=orc.NS_B, c=orc.NS_C, eps=0.0):
        return real_ns(M, steps, a, b, 0.0, eps)

    def ns_wrong_sign(M, steps=5, a=orc.NS_A, b=orc.NS_B, c=orc.NS_C, eps=0.0):
        return real_ns(M, steps, a, -b, c, eps)

    def ns_transposed_gram(M, steps=5, a=orc.NS_A, b=orc.NS_B, c=orc.NS_C, eps=0.0):
        M = np.asarray(M, dtype=np.float64)
        den = np.sqrt(np.sum(M * M)) + eps
        X = M / den if den else np.zeros_like(M)
        for _ in range(steps):
            S = X.T @ X            # wrong side for the left-multiplied form
            if S.shape[0] != X.shape[0]:
                S = np.resize(S, (X.shape[0], X.shape[0]))
            X = a * X + b * (S @ X) + c * (S @ (S @ X))
        return X

    def ns_spectral_norm(M, steps=5, a=orc.NS_A, b=orc.NS_B, c=orc.NS_C, eps=0.0):
        # normalises by the spectral norm instead of the Frobenius norm
        X = np.asarray(M, dtype=np.float64) / max(np.linalg.norm(M, 2), 1e-300)
        for _ in range(steps):
            S = X @ X.T
            X = a * X + b * (S @ X) + c * (S @ (S @ X))
        return X

    for bad in (ns_dropped_quintic, ns_wrong_sign, ns_transposed_gram, ns_spectral_norm):
        monkeypatch.setattr(orc, "newton_schulz", bad)
        assert not _pins_pass(), bad.__name__
    monkeypatch.setattr(orc, "newton_schulz", real_ns)

    def elem_no_roll(self, G, hp):
        keep = self.G_prev.copy()
        M = real_elem(self, G, hp)
        self.G_prev = keep
        return M

    def elem_momentum_on_raw_gradient(self, G, hp):
        G = np.asarray(G, dtype=np.float64)
        D = G - self.G_prev
        self.A = hp.beta_a * self.A + (1 - hp.beta_a) * D
        self.G_tilde = G + hp.alpha * self.A
        self.M = hp.momentum * self.M + G          # acceleration dropped from the momentum
        self.G_prev = G.copy()
        self.k += 1
        return self.M

    def elem_ema_damped_momentum(self, G, hp):
        G = np.asarray(G, dtype=np.float64)
        D = G - self.G_prev
        self.A = hp.beta_a * self.A + (1 - hp.beta_a) * D
        self.G_tilde = G + hp.alpha * self.A
        self.M = hp.momentum * self.M + (1 - hp.momentum) * self.G_tilde   # EMA form is not Eq. muon_momentum
        self.G_prev = G.copy()
        self.k += 1
        return self.M

    def elem_diff_sign(self, G, hp):
        G = np.asarray(G, dtype=np.float64)
        D = self.G_prev - G
        self.A = hp.beta_a * self.A + (1 - hp.beta_a) * D
        self.G_tilde = G + hp.alpha * self.A
        self.M = hp.momentum * self.M + self.G_tilde
        self.G_prev = G.copy()
        self.k += 1
        return self.M

    def elem_one_buffer_carry_without_square(self, G, hp):
        if self.accel_form != "one_buffer":
            return real_elem(self, G, hp)
        G = np.asarray(G, dtype=np.float64)
        self.A = self.C + (1 - hp.beta_a) * G
        self.G_tilde = G + hp.alpha * self.A
        self.M = hp.momentum * self.M + self.G_tilde
        self.C = hp.beta_a * self.A - G            # the carried gradient term lost its (1 - beta_a)
        self.k += 1
        return self.M

    def elem_bf16_rounds_a_before_use(self, G, hp):
        if self.state_dtype != "bf16" or self.accel_form != "two_buffer":
            return real_elem(self, G, hp)
        G = np.asarray(G, dtype=np.float64)
        D = G - self.G_prev
        self.A = orc.round_to_bf16(hp.beta_a * self.A + (1 - hp.beta_a) * D)   # rounded before it feeds G~
        self.G_tilde = G + hp.alpha * self.A
        self.M = hp.momentum * self.M + self.G_tilde
        self.G_prev = orc.round_to_bf16(G)
        self.k += 1
        return self.M

    def elem_bf16_diff_against_unrounded_gradient(self, G, hp):
        if self.state_dtype != "bf16" or self.accel_form != "two_buffer":
            return real_elem(self, G, hp)
        G = np.asarray(G, dtype=np.float64)
        exact_prev = getattr(self, "_exact_prev", np.zeros_like(G))
        D = G - exact_prev                             # as if G_{k-1} had been kept in full precision
        self.A = hp.beta_a * self.A + (1 - hp.beta_a) * D
        self.G_tilde = G + hp.alpha * self.A
        self.M = hp.momentum * self.M + self.G_tilde
        self._exact_prev = G.copy()
        self.A = orc.round_to_bf16(self.A)
        self.G_prev = orc.round_to_bf16(G)
        self.k += 1
        return self.M

    def elem_bf16_rounds_momentum_too(self, G, hp):
        M = real_elem(self, G, hp)
        if self.state_dtype == "bf16":
            self.M = orc.round_to_bf16(self.M)         # M stays full precision in MONA-Lite
        return self.M

    for bad in (elem_no_roll, elem_momentum_on_raw_gradient, elem_ema_damped_momentum, elem_diff_sign,
                elem_one_buffer_carry_without_square, elem_bf16_rounds_a_before_use,
                elem_bf16_diff_against_unrounded_gradient, elem_bf16_rounds_momentum_too):
        monkeypatch.setattr(MonaOracle, "elementwise", bad)
        assert not _pins_pass(), bad.__name__
    monkeypatch.setattr(MonaOracle, "elementwise", real_elem)

    monkeypatch.setattr(orc, "update_scale", lambda m, n, g=0.2: g * math.sqrt(min(m, n)))
    assert not _pins_pass()
    monkeypatch.setattr(orc, "update_scale", real_scale)

    def step_decay_on_new_w(self, W, G, hp):
        W = np.asarray(W, dtype=np.float64)
        M = self.elementwise(G, hp)
        self.norm = float(np.sqrt(np.sum(M * M)))
        self.O = orc.newton_schulz(M, hp.ns_steps, hp.ns_a, hp.ns_b, hp.ns_c, hp.ns_eps)
        gamma = orc.update_scale(self.shape[0], self.shape[1], hp.gamma_coeff)
        W1 = W - hp.lr * gamma * self.O
        return W1 - hp.lr * hp.weight_decay * W1      # decays the updated weights

    monkeypatch.setattr(MonaOracle, "step", step_decay_on_new_w)
    assert not _pins_pass()
    monkeypatch.undo()
    assert _pins_pass()
