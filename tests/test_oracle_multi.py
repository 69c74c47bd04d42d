"""Pins of the oracle's q-direction step (Eq. 2 with q > 1, then Eq. 3), the linear-decay step size of the
hyperparameter table, and the replay of a run from its (seed, coefficient) log.  CPU only."""
import numpy as np

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def _linear_cfg(K, N):
    # one linear layer, no quantizer anywhere: the loss mean((X W^T - T)^2) is exactly quadratic in W
    return orc.Config(orc.ARCH_LINEAR, d_model=K, d_ffn=N, w_bits=0, w_group=0, a_bits=16, act_dtype=0)


def _grad_mse(W, X, T):
    Y = X.astype(np.float64) @ W.astype(np.float64).T
    return 2.0 * (Y - T).T @ X.astype(np.float64) / Y.size


def test_q1_is_the_single_direction_step_bit_for_bit():
    cfg = orc.Config(orc.ARCH_LINEAR, d_model=64, d_ffn=16, w_bits=4, w_group=32, a_bits=8, act_dtype=0)
    W = synth.weights((16, 64), 1)
    X, T = synth.activations((8, 64), 2), synth.activations((8, 16), 3)
    a, b = [W.copy()], [W.copy()]
    r1 = orc.zo_step(cfg, a, 5, 1e-3, 1e-2, x=X, target=T)
    rq = orc.zo_step_multi(cfg, b, [5], 1e-3, 1e-2, x=X, target=T)
    assert rq == [r1] and np.array_equal(a[0], b[0])


def test_average_of_directions_on_a_quadratic():
    # Q = identity, quadratic loss: g_i = u_i . grad L exactly, all directions taken at the same W, so
    # (W0 - W1) / eta = (1/q) sum_i (u_i . grad) u_i.  eta is large enough that evaluating direction 2 at
    # an already updated W, a missing 1/q, a wrong sign or a swapped seed would each miss by far more
    # than the tolerance.
    K, N, M = 12, 5, 7
    cfg = _linear_cfg(K, N)
    W0 = synth.weights((N, K), 11, scale=0.5)
    X, T = synth.activations((M, K), 12), synth.activations((M, N), 13)
    G = _grad_mse(W0, X, T)
    seeds = [3, 10, 4, 77]
    lr = 0.05
    p = [W0.copy()]
    res = orc.zo_step_multi(cfg, p, seeds, 1e-3, lr, x=X, target=T)
    est = np.zeros_like(G)
    for s, (_, _, g) in zip(seeds, res):
        u = orc.normal(s, 0, N * K).astype(np.float64).reshape(N, K)
        assert abs(float(g) - np.sum(u * G)) <= 2e-3 * max(1.0, abs(np.sum(u * G)))      # fp32 losses / 2 eps
        est += np.sum(u * G) * u / len(seeds)
    got = (W0.astype(np.float64) - p[0]) / lr
    assert np.abs(got - est).max() <= 3e-3 * np.abs(est).max()
    # sequential evaluation (direction i at the W updated by directions < i) is a different, measurably distinct result
    ps = [W0.copy()]
    for s in seeds:
        orc.zo_step(cfg, ps, s, 1e-3, lr / len(seeds), x=X, target=T)
    assert np.abs((W0.astype(np.float64) - ps[0]) / lr - est).max() > 3e-2 * np.abs(est).max()


def test_error_of_the_average_falls_like_one_over_q():
    # Prop. 1(ii): the mean squared error carries the factor 1/q.  On a quadratic with Q = identity the estimate
    # (1/q) sum (u_i . G) u_i has MSE |G|^2 (d + 1) / q exactly (E (u.G)^2 |u|^2 = |G|^2 (d + 2)).
    K, N, M = 4, 2, 3
    d = K * N
    cfg = _linear_cfg(K, N)
    W0 = synth.weights((N, K), 21, scale=0.5)
    X, T = synth.activations((M, K), 22), synth.activations((M, N), 23)
    G = _grad_mse(W0, X, T)
    lr = 1e-2
    mse = {}
    for q in (1, 4):
        n = 1600 // q
        acc = 0.0
        for t in range(n):
            p = [W0.copy()]
            orc.zo_step_multi(cfg, p, [1000 * q + t * q + i for i in range(q)], 1e-3, lr, x=X, target=T)
            acc += np.sum(((W0.astype(np.float64) - p[0]) / lr - G) ** 2)
        mse[q] = acc / n
        want = np.sum(G * G) * (d + 1) / q
        # relative standard error of the MSE estimate over n draws is about sqrt((2 + 12/d) / n); 4.5 sigma
        assert abs(mse[q] - want) <= 4.5 * np.sqrt((2 + 12.0 / d) / n) * want + 0.02 * want, (q, mse[q], want)
    assert 2.8 < mse[1] / mse[4] < 5.6


def test_update_applies_the_terms_in_seed_order():
    # the multi-direction update is the composition of the pinned single-direction updates, in order
    cfg = _linear_cfg(16, 8)
    W0 = synth.weights((8, 16), 31)
    X, T = synth.activations((4, 16), 32), synth.activations((4, 8), 33)
    seeds = [9, 2, 5]
    p = [W0.copy()]
    res = orc.zo_step_multi(cfg, p, seeds, 1e-3, 0.3, x=X, target=T)
    w = W0.copy()
    lrq = np.float32(np.float32(0.3) / np.float32(3))
    for s, (_, _, g) in zip(seeds, res):
        orc.update(w, s, 0, orc.coeff(lrq, g))
    assert np.array_equal(w, p[0])


def test_linear_decay_schedule():
    lr0, T = np.float32(5e-7), 10000
    assert orc.lr_linear_decay(lr0, 0, T) == lr0
    assert orc.lr_linear_decay(lr0, T // 2, T) == np.float32(float(lr0) * 0.5)
    assert orc.lr_linear_decay(lr0, T - 1, T) == np.float32(float(lr0) / T)
    v = [float(orc.lr_linear_decay(lr0, t, T)) for t in range(0, T, 997)]
    assert all(a > b for a, b in zip(v, v[1:])) and v[-1] > 0
    assert orc.lr_linear_decay(1.0, 3, 4) == np.float32(0.25)


def test_replay_from_the_seed_and_coefficient_log():
    # the forward passes only produce one scalar per direction; (seed, c) per step reproduces the run exactly
    cfg = orc.Config(orc.ARCH_LINEAR, d_model=32, d_ffn=8, w_bits=4, w_group=32, a_bits=16, act_dtype=0)
    W0 = synth.weights((8, 32), 41)
    X, T = synth.activations((4, 32), 42), synth.activations((4, 8), 43)
    p, log = [W0.copy()], []
    for t in range(6):
        lr = orc.lr_linear_decay(1e-2, t, 6)
        _, _, g = orc.zo_step(cfg, p, 100 + t, 1e-3, lr, x=X, target=T)
        log.append((100 + t, orc.coeff(lr, g)))
    w = W0.copy()
    for seed, c in log:
        orc.update(w, seed, 0, c)
    assert np.array_equal(w, p[0]) and not np.array_equal(w, W0)
