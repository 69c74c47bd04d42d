"""Pins of the oracle's adaptive weight quantizer (Eq. 5: learnable step, zero point, clipping
coefficients) and channel-wise smoothing (Eq. 4), and of their wiring into the model and the ZO step
(three learning-rate groups: Appendix, hyperparameter table)."""
import numpy as np

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def test_eq5_hand_worked_group():
    # 2 bits (Q_P = 3), step 1/2, zero point 1
    x = np.array([-1.0, -0.5, 0.0, 0.26, 0.74, 2.0], np.float32)
    codes, xhat = orc.quant_group_learned(x, 2, 0.5, 1.0, 0.0, 1.0)
    assert codes.tolist() == [0, 0, 1, 2, 2, 3]
    assert xhat.tolist() == [-0.5, -0.5, 0.0, 0.5, 0.5, 1.0]
    # clipping coefficients 1/3 and 2/3: codes confined to [1, 2]
    codes, xhat = orc.quant_group_learned(x, 2, 0.5, 1.0, 1.0 / 3.0, 2.0 / 3.0)
    assert codes.tolist() == [1, 1, 1, 2, 2, 2]
    assert xhat.tolist() == [0.0, 0.0, 0.0, 0.5, 0.5, 0.5]
    # a real-valued zero point acts through its rounding; bounds stay inside [0, Q_P] and ordered
    c1, _ = orc.quant_group_learned(x, 2, 0.5, 1.4, -0.3, 1.7)
    assert c1.tolist() == [0, 0, 1, 2, 2, 3]
    c2, h2 = orc.quant_group_learned(x, 2, 0.5, 1.0, 0.9, 0.2)       # crossed bounds collapse onto the lower one
    assert set(c2.tolist()) == {3} and np.all(h2 == 1.0)


def test_eq5_matches_literal_formula_except_ties():
    rng = synth.rng(601)
    bad = 0
    for t in range(300):
        bits = int(rng.integers(2, 9))
        qp = 2 ** bits - 1
        x = (rng.standard_normal(64) * 0.05).astype(np.float32)
        step = np.float32(np.ptp(x) / qp * rng.uniform(0.7, 1.3))
        zp = np.float32(rng.uniform(0, qp))
        alpha, beta = np.float32(rng.uniform(0, 0.3)), np.float32(rng.uniform(0.7, 1.0))
        codes, xhat = orc.quant_group_learned(x, bits, step, zp, alpha, beta)
        r = x.astype(np.float64) / np.float64(step)
        lit = np.clip(np.rint(r) + np.rint(np.float64(zp)), np.rint(np.float64(alpha) * qp), np.rint(np.float64(beta) * qp))
        tie = np.abs(np.abs(r - np.floor(r)) - 0.5) < 1e-5
        bad += int(np.sum((codes != lit) & ~tie))
        assert np.allclose(xhat, (codes - np.rint(np.float64(zp))) * np.float64(step), rtol=1e-6, atol=0)
    assert bad == 0


def test_initial_parameters_reproduce_the_dynamic_quantizer():
    W = synth.weights((24, 256), 602)
    for bits, g in ((4, 64), (2, 128), (4, 0)):
        step, zp, alpha, beta = orc.init_learned(W, bits, g)
        dyn = orc.fakequant_weight(W, bits, g)
        assert np.array_equal(step, dyn["step"]) and np.array_equal(zp, dyn["zp"].astype(np.float32))
        assert np.all(alpha == 0) and np.all(beta == 1)
        got = orc.fakequant_weight_learned(W, bits, g, step, zp, alpha, beta)
        assert np.array_equal(got["codes"], dyn["codes"]) and np.array_equal(got["what"], dyn["what"])
    # tighter clipping saturates the extremes and only them
    step, zp, alpha, beta = orc.init_learned(W, 4, 64)
    got = orc.fakequant_weight_learned(W, 4, 64, step, zp, alpha + 0.2, beta - 0.2)
    dyn = orc.fakequant_weight(W, 4, 64)
    assert got["codes"].min() == 3 and got["codes"].max() == 12
    inside = (dyn["codes"] >= 3) & (dyn["codes"] <= 12)
    assert np.array_equal(got["codes"][inside], dyn["codes"][inside])


def test_eq4_is_an_exact_reparametrisation_without_quantization():
    rng = synth.rng(603)
    X = synth.activations((40, 96), 604)
    W = synth.weights((56, 96), 605, scale=1.0)
    s = (1.0 + rng.uniform(-0.4, 0.6, 96)).astype(np.float32)
    delta = (0.3 * rng.standard_normal(96)).astype(np.float32)
    inv_s = (np.float32(1.0) / s).astype(np.float32)
    xbar = orc.smooth_act(X, delta, inv_s)
    assert np.array_equal(xbar, ((X - delta[None, :]) * inv_s[None, :]).astype(np.float32))
    wbar = W.astype(np.float64) * s.astype(np.float64)[None, :]
    y = xbar.astype(np.float64) @ wbar.T + (W.astype(np.float64) @ delta.astype(np.float64))[None, :]
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.max(np.abs(y - ref)) < 1e-5 * np.max(np.abs(ref))
    # the weight operand really is s (.) W along the in-feature axis
    got = orc.fakequant_weight_learned(W, 8, 96, *[a for a in orc.init_learned(W, 8, 96, s)], scale=s)["what"]
    assert np.max(np.abs(got - wbar)) <= 0.5001 * np.max(orc.init_learned(W, 8, 96, s)[0])


def _model(cfg_kw, seed):
    cfg = orc.Config(orc.ARCH_OPT, n_layers=2, d_model=64, n_heads=2, d_ffn=128, vocab=101, max_seq=12,
                     w_bits=4, w_group=32, a_bits=8, act_dtype=0, **cfg_kw)
    params = synth.model_params(orc.param_shapes(cfg), seed)
    return cfg, params


def test_model_with_initial_learned_parameters_equals_the_dynamic_model_at_eps_zero():
    ids = synth.token_ids(2, 12, 101, 9)
    cfg0, p0 = _model({}, 606)
    base = orc.forward(cfg0, p0, ids=ids, seed=1, eps_signed=0.0)
    for kw in (dict(learn_clip=1), dict(learn_smooth=1), dict(learn_clip=1, learn_smooth=1)):
        cfg, p = _model(kw, 606)
        assert len(p) > len(p0) and all(np.array_equal(a, b) for a, b in zip(p0, p))
        orc.init_learned_params(cfg, p)
        assert orc.forward(cfg, p, ids=ids, seed=1, eps_signed=0.0) == base
        # a perturbed forward differs from the dynamic one (static parameters, perturbed themselves)
        assert orc.forward(cfg, p, ids=ids, seed=1, eps_signed=1e-3) != orc.forward(cfg0, p0, ids=ids, seed=1, eps_signed=1e-3)


def test_smoothing_changes_what_the_activation_quantizer_sees_but_not_the_float_function():
    ids = synth.token_ids(2, 12, 101, 9)
    rng = synth.rng(607)
    # 8-bit weights per channel and A16: nearly the float model; a non-trivial (s, delta) must leave the loss almost unchanged
    kw = dict(n_layers=1, d_model=64, n_heads=2, d_ffn=128, vocab=101, max_seq=12, w_bits=8, w_group=0, a_bits=16, act_dtype=0)
    cfg = orc.Config(orc.ARCH_OPT, learn_smooth=1, **kw)
    p = synth.model_params(orc.param_shapes(cfg), 608)
    orc.init_learned_params(cfg, p)
    base = orc.forward(cfg, p, ids=ids)
    for i, (name, shape, _) in enumerate(orc.param_shapes(cfg)):
        if name.endswith(".sm_s"):
            p[i][...] = (1.0 + rng.uniform(-0.3, 0.5, shape)).astype(np.float32)
        if name.endswith(".sm_delta"):
            p[i][...] = (0.2 * rng.standard_normal(shape)).astype(np.float32)
    moved = orc.forward(cfg, p, ids=ids)
    assert moved != base and abs(moved - base) < 2e-3 * abs(base)


def test_zo_step_uses_one_coefficient_per_learning_rate_group():
    ids = synth.token_ids(2, 12, 101, 9)
    cfg, p = _model(dict(learn_clip=1, learn_smooth=1), 609)
    orc.init_learned_params(cfg, p)
    before = [a.copy() for a in p]
    lrs = (1e-3, 5e-3, 2e-2)
    lp, lm, g = orc.zo_step(cfg, p, seed=11, eps=1e-3, lr=lrs[0], ids=ids, lr_smooth=lrs[1], lr_clip=lrs[2])
    assert g != 0
    groups = orc.param_groups(cfg)
    assert sorted(set(groups)) == [0, 1, 2]
    for i, (w0, w1) in enumerate(zip(before, p)):
        c = orc.coeff(np.float32(lrs[groups[i]]), g)
        assert np.array_equal(w1, orc.update(w0.copy(), 11, i, c))
        z = orc.normal(11, i, w0.size).reshape(w0.shape)
        big = np.abs(z) > 0.5
        assert np.allclose((w1 - w0)[big] / -c, z[big], rtol=2e-2)
