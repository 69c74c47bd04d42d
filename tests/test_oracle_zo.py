"""Pins for the oracle's estimator and update (Eq. 2 with q = 1, Eq. 3), CPU only:
closed forms on a quadratic, the 1-D Gaussian-smoothed quantized objective of the
theory appendix (unbiasedness, Prop. 1(i); second-moment bound, Prop. 1(ii))."""
import numpy as np
from scipy import stats

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def _spsa(loss, w, seed, eps, tensor_id=0):
    eps = np.float32(eps)
    lp = np.float32(loss(orc.perturb(w, seed, tensor_id, eps)))
    lm = np.float32(loss(orc.perturb(w, seed, tensor_id, -eps)))
    return orc.projected_grad(lp, lm, eps)


def test_quadratic_closed_form():
    # L = 1/2 w^T A w + b^T w, Q = identity: (L(w+eps z) - L(w-eps z)) / 2eps = z^T (A w + b) exactly
    d = 48
    r = synth.rng(1)
    A = r.standard_normal((d, d)); A = A @ A.T / d
    b = r.standard_normal(d)
    w = synth.activations((d,), 2)
    loss = lambda v: 0.5 * v.astype(np.float64) @ A @ v.astype(np.float64) + b @ v.astype(np.float64)
    for seed in range(5):
        z = orc.normal(seed, 0, d).astype(np.float64)
        want = z @ (A @ w.astype(np.float64) + b)
        got = _spsa(loss, w, seed, 1e-2)
        # fp32 storage of the two losses limits the quotient: |L| * 2^-24 / eps
        assert abs(got - want) <= 2e-3 * max(1.0, abs(want)), (seed, got, want)


def test_smooth_loss_error_shrinks_like_eps_squared():
    d = 16
    w = synth.activations((d,), 3).astype(np.float64) * 0.3
    z = orc.normal(4, 0, d).astype(np.float64)
    f = lambda v: np.sum(np.sin(v))
    grad = z @ np.cos(w)
    errs = []
    for eps in (0.2, 0.1, 0.05):
        est = (f(w + eps * z) - f(w - eps * z)) / (2 * eps)      # same formula in exact arithmetic
        errs.append(abs(est - grad))
    assert 3.0 < errs[0] / errs[1] < 5.0 and 3.0 < errs[1] / errs[2] < 5.0
    # and the oracle's fp32 path agrees with that formula
    got = _spsa(lambda v: f(v.astype(np.float64)), w.astype(np.float32), 4, 0.05)
    est = (f(w.astype(np.float32) + 0.05 * z) - f(w.astype(np.float32) - 0.05 * z)) / 0.1
    assert abs(got - est) < 1e-4 * max(1, abs(est))


def test_projected_grad_and_coeff_arithmetic():
    assert orc.projected_grad(np.float32(2.0), np.float32(1.0), np.float32(0.25)) == np.float32(2.0)
    assert orc.projected_grad(np.float32(1.0), np.float32(2.0), np.float32(0.25)) == np.float32(-2.0)
    lp, lm, eps = np.float32(10.400001), np.float32(10.399), np.float32(1e-3)
    want = (float(lp) - float(lm)) / (2 * float(eps))
    assert orc.projected_grad(lp, lm, eps) == np.float32(want)
    assert orc.coeff(np.float32(1e-4), np.float32(3.0)) == np.float32(float(np.float32(1e-4)) * 3.0)


def test_update_is_seeded_axpy():
    w0 = synth.weights((1000,), 5)
    z = orc.normal(31, 7, 1000)
    # zero coefficient: identity
    assert np.array_equal(orc.update(w0.copy(), 31, 7, np.float32(0.0)), w0)
    # (w1 - w0) / (-c) reproduces z to rounding
    c = np.float32(1e-2)
    w1 = orc.update(w0.copy(), 31, 7, c)
    assert np.abs((w1.astype(np.float64) - w0) / (-float(c)) - z).max() < 1e-4
    want = (w0.astype(np.float64) - float(c) * z.astype(np.float64))
    assert np.abs(w1 - want).max() <= 2 ** -24 * np.abs(want).max() * 1.01
    # linear in c; the sign is descent (minus)
    w2 = orc.update(w0.copy(), 31, 7, np.float32(2e-2))
    assert np.allclose((w2 - w0.astype(np.float64)), 2 * (w1 - w0.astype(np.float64)), atol=1e-7)
    # plus then minus restores to rounding
    w3 = orc.update(orc.update(w0.copy(), 31, 7, c), 31, 7, -c)
    assert np.abs(w3 - w0).max() <= 2 ** -22 * np.abs(w0).max()


def test_step_on_quadratic_descends_in_expectation():
    # one full step with Q = identity on L = 1/2 |w|^2: E[w1] = w0 - lr * w0 (E[z z^T] = I)
    d = 8
    w0 = np.ones(d, np.float32)
    acc = np.zeros(d)
    n = 4000
    lr = 0.1
    for seed in range(n):
        w = w0.copy()
        g = _spsa(lambda v: 0.5 * np.sum(v.astype(np.float64) ** 2), w, seed, 1e-3)
        orc.update(w, seed, 0, orc.coeff(np.float32(lr), g))
        acc += w
    mean = acc / n
    # Var of one coordinate of g z is about (d + 1) * |w0|^2-ish; allow 5 sigma
    assert np.abs(mean - (1 - lr) * w0).max() < 5 * lr * np.sqrt((d + 2.0) / n)


# ---- 1-D quantized objective of the theory appendix ---------------------------------------
def _fixed_step_quant(w, lo, hi, bits):
    """Uniform quantizer with a fixed step, built from the oracle's group quantizer by adding two
    anchors that pin min and max: step = (hi - lo) / Q_P, thresholds at (k + 1/2) * step."""
    _, _, _, xhat = orc.quant_group(np.array([lo, w, hi], np.float32), bits)
    return float(xhat[1])


def test_unbiased_for_gaussian_smoothed_quantized_objective_1d():
    # d = 1, L = G * Q(W).  f_eps(W) = G E[Q(W + eps U)], so
    # grad f_eps(W) = (G step / eps) * sum_k phi((tau_k - W) / eps) over the thresholds tau_k.
    # Anchors -1.5 / 1.5 with 2 bits: step 1, zero-point 2, Q(w) = round(w) clamped to [-2, 1];
    # thresholds at -1.5, -0.5, 0.5 (the one at 1.5 is removed by the clamp).
    G, bits, lo, hi = 3.0, 2, -1.5, 1.5
    step = (hi - lo) / (2 ** bits - 1)
    th = np.array([-1.5, -0.5, 0.5])
    for W, eps in ((0.07, 0.25), (0.45, 0.25), (-0.9, 0.1)):
        n = 60000
        est = np.empty(n)
        w = np.array([W], np.float32)
        e = np.float32(eps)
        for seed in range(n):
            z = float(orc.z_at(seed, 0, 0))
            lp = np.float32(G * _fixed_step_quant(float(orc.perturb(w, seed, 0, e)[0]), lo, hi, bits))
            lm = np.float32(G * _fixed_step_quant(float(orc.perturb(w, seed, 0, -e)[0]), lo, hi, bits))
            est[seed] = float(orc.projected_grad(lp, lm, e)) * z
        want = G * step / eps * np.sum(stats.norm.pdf((th - W) / eps))
        se = est.std() / np.sqrt(n)
        assert abs(est.mean() - want) < 4.5 * se + 1e-3 * abs(want), (W, eps, est.mean(), want, se)
        # Prop. 1(ii) with d = q = 1: E|g - grad f|^2 <= 2 G^2 * 3 + G^2 step^2 / (2 eps^2)
        bound = 6 * G * G + G * G * step * step / (2 * eps * eps)
        assert np.mean((est - want) ** 2) <= bound


def test_far_from_thresholds_the_estimate_vanishes():
    # distance to the nearest threshold r = 0.5 * step, eps small: the Lemma-2 bound is ~ 0
    G, bits, lo, hi = 1.0, 2, -1.5, 1.5
    w = np.array([0.0], np.float32)                     # cell centre; nearest thresholds at +-0.5
    eps = np.float32(0.05)                              # t = r / eps = 10
    total = 0.0
    for seed in range(2000):
        lp = np.float32(G * _fixed_step_quant(float(orc.perturb(w, seed, 0, eps)[0]), lo, hi, bits))
        lm = np.float32(G * _fixed_step_quant(float(orc.perturb(w, seed, 0, -eps)[0]), lo, hi, bits))
        total += abs(float(orc.projected_grad(lp, lm, eps)))
    assert total == 0.0
