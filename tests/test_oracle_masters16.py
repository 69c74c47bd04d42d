"""Pins of the oracle's binary16 master weights (2 bytes per parameter, what the memory table of the efficiency
section implies): the forward reads the stored value exactly; the update of Eq. 3 is one fp32 fma and one
rounding to binary16, to nearest even or stochastic.  CPU only."""
import numpy as np

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def _f16(bits):
    return np.array([bits], np.uint16).view(np.float16)[0]


def test_stochastic_rounding_brackets_and_keeps_representable_values():
    r = synth.rng(301)
    xs = np.concatenate([r.standard_normal(400).astype(np.float32) * np.float32(0.02),
                         r.standard_normal(200).astype(np.float32) * np.float32(3e-5),      # binary16 subnormals
                         np.array([0.0, -0.0, 1.0, -1.0, 6.1e-5, -5.96e-8, 2.0 ** -25, -2.0 ** -26, 65504.0, 1e-30],
                                  np.float32)])
    for x in xs:
        for rr in (0, 1, 2 ** 23, 2 ** 24 - 1, int(r.integers(0, 2 ** 24))):
            h = orc.f32_to_f16_stochastic(x, rr)
            v = float(_f16(h))
            near = float(np.float16(x))                              # numpy's nearest-even conversion
            if float(np.float32(near)) == float(x):
                assert v == float(x)                                 # representable: unchanged whatever r
                continue
            lo = float(np.nextafter(np.float16(near), np.float16(-np.inf))) if near > x else near
            hi = near if near > x else float(np.nextafter(np.float16(near), np.float16(np.inf)))
            assert lo < float(x) < hi and v in (lo, hi), (x, rr, v, lo, hi)


def test_stochastic_rounding_probability_is_the_fraction():
    # x = lo + frac * ulp: up exactly for the r below frac * 2^24, so P(up) = ceil(frac 2^24) / 2^24
    lo, ulp = 1.0, 2.0 ** -10
    for k in (1, 3, 4096, 8191):                                     # frac = k / 8192: 13 dropped bits
        x = np.float32(lo + k / 8192.0 * ulp)
        thr = k * 2048                                               # frac * 2^24
        assert float(_f16(orc.f32_to_f16_stochastic(x, thr - 1))) == lo + ulp
        assert float(_f16(orc.f32_to_f16_stochastic(x, thr))) == lo
        assert float(_f16(orc.f32_to_f16_stochastic(x, 0))) == lo + ulp
    # negative values: "up" is toward +infinity
    x = np.float32(-(1.0 + 0.25 * ulp))                              # lo = -(1 + ulp), hi = -1, frac = 0.75
    assert float(_f16(orc.f32_to_f16_stochastic(x, int(0.75 * 2 ** 24) - 1))) == -1.0
    assert float(_f16(orc.f32_to_f16_stochastic(x, int(0.75 * 2 ** 24)))) == -(1.0 + ulp)
    # across zero: |x| below half the smallest subnormal still reaches it with probability x / 2^-24
    x = np.float32(2.0 ** -27)
    assert float(_f16(orc.f32_to_f16_stochastic(x, 2 ** 21 - 1))) == 2.0 ** -24
    assert float(_f16(orc.f32_to_f16_stochastic(x, 2 ** 21))) == 0.0


def test_round_bits_stream_is_uniform_and_apart_from_the_perturbation_stream():
    n = 40000
    r = np.array([orc.round_bits(5, 3, i) for i in range(n)], np.float64)
    assert r.max() < 2 ** 24 and r.min() >= 0
    u = r / 2 ** 24
    assert abs(u.mean() - 0.5) < 4 / np.sqrt(12 * n) and abs(u.var() - 1 / 12) < 0.004
    words = orc.philox_words(5, 3, n)                               # the perturbation stream's words
    assert np.mean((words >> 8) == r.astype(np.uint32)) < 1e-3
    assert orc.round_bits(5, 3, 7) == orc.round_bits(5, 3, 7) != orc.round_bits(6, 3, 7)


def test_update_nearest_even_matches_numpy_and_loses_small_steps():
    w0 = synth.weights((5000,), 302).astype(np.float16)
    z = orc.normal(9, 4, 5000).astype(np.float64)
    c = np.float32(3e-3)
    w1 = orc.update(w0.copy(), 9, 4, c)
    x = np.float32(w0.astype(np.float32)) - np.float32(c) * z          # fp64 value of the fma argument
    want = np.array([np.float32(v) for v in x]).astype(np.float16)     # fp32 rounding of the fma, then binary16
    assert np.mean(w1 != want) < 2e-3                                  # double rounding differs from one fma + one rounding only on rare ties
    assert np.abs(w1.astype(np.float64) - x).max() <= 2.0 ** -11 * np.abs(x).max() * 1.01
    # a step far below half the spacing of binary16 is rounded away entirely: the hazard of 16-bit masters
    big = np.full(4096, 1.0, np.float16)
    assert np.array_equal(orc.update(big.copy(), 9, 4, np.float32(1e-5)), big)
    # c = 0 is the identity in both modes
    assert np.array_equal(orc.update(w0.copy(), 9, 4, np.float32(0.0)), w0)
    assert np.array_equal(orc.update(w0.copy(), 9, 4, np.float32(0.0), stochastic=True), w0)


def test_stochastic_update_keeps_the_expected_step():
    # masters at 1.0 (spacing 2^-10 above, 2^-11 below), c u ~ 1e-5: nearest-even loses every step, the stochastic
    # rounding moves a few elements by a whole spacing so that the mean step is -c u
    n = 200000
    w0 = np.full(n, 1.0, np.float16)
    c = np.float32(1e-5)
    z = orc.normal(11, 2, n).astype(np.float64)
    w1 = orc.update(w0.copy(), 11, 2, c, stochastic=True)
    step = w1.astype(np.float64) - 1.0
    assert set(np.unique(step)).issubset({0.0, 2.0 ** -10, -2.0 ** -11})
    # per-element variance of the rounding is at most ulp * |c u|; 5 sigma on the sum
    tol = 5 * np.sqrt(np.sum(2.0 ** -10 * np.abs(float(c) * z)))
    assert abs(np.sum(step) - np.sum(-float(c) * z)) < tol
    # correlation with the direction: sum(step * u) ~ -c sum(u^2)
    tol2 = 5 * np.sqrt(np.sum(2.0 ** -10 * np.abs(float(c) * z) * z * z))
    assert abs(np.sum(step * z) + float(c) * np.sum(z * z)) < tol2
    # same seed, same result; another seed, another rounding pattern
    assert np.array_equal(w1, orc.update(w0.copy(), 11, 2, c, stochastic=True))


def test_step_with_binary16_masters_reads_the_stored_values():
    # the forward of a model whose masters are binary16 equals the forward of the same values held in fp32
    cfg = orc.Config(orc.ARCH_LLAMA, n_layers=1, d_model=32, n_heads=2, d_ffn=64, vocab=64, max_seq=8, w_bits=4, w_group=32,
                     a_bits=8, act_dtype=0)
    p32 = synth.model_params(orc.param_shapes(cfg), 303)
    p16 = [p.astype(np.float16) for p in p32]
    as32 = [p.astype(np.float32) for p in p16]
    ids = synth.token_ids(2, 8, 64, 304)
    assert orc.forward(cfg, p16, ids=ids, seed=3, eps_signed=1e-3) == orc.forward(cfg, as32, ids=ids, seed=3, eps_signed=1e-3)
    lp, lm, g = orc.zo_step(cfg, p16, 3, 1e-3, 1e-2, ids=ids)
    lp2, lm2, g2 = orc.zo_step(cfg, as32, 3, 1e-3, 1e-2, ids=ids)
    assert (lp, lm, g) == (lp2, lm2, g2)
    for a, b in zip(p16, as32):
        assert a.dtype == np.float16 and np.array_equal(a, b.astype(np.float16))   # one rounding of the same fp32 result


def test_multi_direction_update_rounds_once():
    # q terms in fp32, one rounding: for q = 1 the same as the single update; for q > 1 not the same as rounding
    # after every term (which loses the small ones), and within one spacing of the exact sum
    w0 = synth.weights((3000,), 305).astype(np.float16)
    seeds, cs = [4, 5, 6], [np.float32(2e-4), np.float32(-1e-4), np.float32(3e-4)]
    for st in (False, True):
        a = orc.update_multi(w0.copy(), seeds[:1], 2, cs[:1], st)
        assert np.array_equal(a, orc.update(w0.copy(), seeds[0], 2, cs[0], st))
    once = orc.update_multi(w0.copy(), seeds, 2, cs)
    seq = w0.copy()
    for s, c in zip(seeds, cs):
        orc.update(seq, s, 2, c)
    assert not np.array_equal(once, seq)
    exact = w0.astype(np.float64) - sum(float(c) * orc.normal(s, 2, 3000).astype(np.float64) for s, c in zip(seeds, cs))
    assert np.all(np.abs(once.astype(np.float64) - exact) <= 2.0 ** -11 * np.abs(exact) + 2.0 ** -25)
    assert np.abs(once.astype(np.float64) - exact).sum() < np.abs(seq.astype(np.float64) - exact).sum()
