"""GPU parity of the projected gradient g = (L+ - L-) / (2 eps) of Eq. 2, the one scalar that drives the update.

g divides the difference of two nearly equal losses by 2 eps = 2e-3, so an absolute loss error is amplified 500 times.
Where activation codes are decided (A8 / A4) a code is taken from an fp32 activation whose last bits differ between
the GPU (fp32 accumulation) and the oracle (fp64): an element that sits on a rounding boundary may come out one code
apart, and that is a different (equally valid) quantized network.  The oracle alone tells which seeded inputs are
free of such elements (`tie_log`: per quantizer call and row, the distance of the closest element to a rounding
boundary, in code units): on those the benchmark spec's tolerance, 1e-3 relative, is asserted outright; the absolute
term is the resolution of an fp32 loss (~4.8e-7 at L ~ 6) divided by 2 eps, times a few roundings.

bf16 storage adds the rounding of every stored activation to 8 bits of mantissa; GPU and oracle round the same
value unless it lies within their ~1e-7 relative disagreement of a bf16 rounding boundary, which happens to about
5e-5 of the stored elements; each such element moves one activation by one bf16 spacing.  g then carries noise that
no implementation detail removes; it is reported over 16 seeds and bounded against that model."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu

TIE_MARGIN = 1e-4      # code units; the GPU's fp32 activations differ from the oracle's by < 4e-5 code units at 8 bits
EPS = 1e-3


def _small_model(arch, act_dtype, a_bits, seed):
    base = dict(n_layers=1, d_model=64, n_heads=2, d_ffn=128, vocab=256, max_seq=8, w_bits=4, w_group=32, a_bits=a_bits)
    ocfg = orc.Config(arch, act_dtype=act_dtype, **base)
    params = synth.model_params(orc.param_shapes(ocfg), 700 + seed)
    params = [p * (3.0 if p.ndim == 2 else 1.0) for p in params]
    ids = synth.token_ids(2, 8, base["vocab"], 800 + seed)
    return base, ocfg, params, ids


def _oracle_pair(ocfg, params, ids, seed):
    """Both forwards of Eq. 2 on the oracle; returns (L+, L-, g, smallest tie margin met in either branch)."""
    ties = []
    lp = orc.forward(ocfg, params, ids=ids, seed=seed, eps_signed=np.float32(EPS), tie_log=ties)
    lm = orc.forward(ocfg, params, ids=ids, seed=seed, eps_signed=np.float32(-EPS), tie_log=ties)
    margin = min((float(m.min()) for m in ties), default=1.0)
    return lp, lm, orc.projected_grad(lp, lm, np.float32(EPS)), margin


@pytest.mark.parametrize("arch", [1, 2])
@pytest.mark.parametrize("a_bits", [8, 4])
def test_g_within_1e3_on_tie_free_inputs(arch, a_bits):
    """fp32 storage, activation codes on: seeded inputs on which the oracle meets no element within TIE_MARGIN of a
    rounding boundary in either branch (found by running the oracle alone over seeds 0, 1, ...).  There L+, L- and g
    are held to the benchmark spec's tolerance."""
    torch, zo = gpu()
    found, flagged = 0, 0
    for seed in range(400):
        base, ocfg, params, ids = _small_model(arch, 0, a_bits, seed)
        lp, lm, g, margin = _oracle_pair(ocfg, params, ids, seed)
        if margin < TIE_MARGIN:
            flagged += 1
            continue
        cfg = zo.make_config(arch, act_dtype=0, **base)
        gp = [to_dev(p, torch) for p in params]
        ctx = zo.Context(cfg, gp, 2, 8)
        out = ctx.zo_step(to_dev(ids, torch), None, 2, 8, seed=seed, eps=EPS, lr=0.0).cpu().numpy()
        ctx.close()
        assert abs(out[0] - lp) <= 1e-5 * abs(lp) and abs(out[1] - lm) <= 1e-5 * abs(lm), (seed, out, lp, lm)
        assert abs(out[2] - g) <= 1e-3 * abs(g) + 1e-3, (seed, out[2], g)
        found += 1
        if found == 6:
            break
    print("arch %d A%d: %d tie-free inputs checked, %d seeds skipped for a flagged tie" % (arch, a_bits, found, flagged))
    assert found == 6


@pytest.mark.parametrize("a_bits", [16, 8])
def test_g_noise_in_bf16_storage(a_bits):
    """bf16 storage (the benchmark's mode): g over 16 seeded steps against the oracle.  Noise model: a stored element
    on which the two sides round differently (probability ~5e-5 each) moves one token's hidden state by one bf16
    spacing (2^-8 relative on one of d coordinates) and with it the mean loss by about |L| 2^-8 / (sqrt(d) B S);
    n such elements per branch give delta g ~ sqrt(2 n) |L| 2^-8 / (sqrt(d) B S 2 eps).  With d = 128, B S = 64,
    |L| ~ 6.3 and n ~ 10 (2e5 stored elements per forward): ~0.1 absolute on |g| of order 1..10; with activation
    codes a differently rounded element can also flip a code (one code unit ~ one bf16 spacing of the row's large
    elements), which doubles the count.  Asserted: losses 1e-3 (the benchmark spec); median |delta g| <= 0.15 and
    max <= 0.6 -- a few times the model, so that a systematic error of the size of one stored tensor's rounding
    (which would shift every seed the same way) fails."""
    torch, zo = gpu()
    B, S = 2, 32
    base = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=256, vocab=512, max_seq=S, w_bits=4, w_group=64, a_bits=a_bits)
    ocfg = orc.Config(1, act_dtype=1, **base)
    cfg = zo.make_config(1, act_dtype=1, **base)
    dg, gs = [], []
    for seed in range(16):
        params = synth.model_params(orc.param_shapes(ocfg), 900 + seed)
        params = [p * (3.0 if p.ndim == 2 else 1.0) for p in params]
        ids = synth.token_ids(B, S, base["vocab"], 950 + seed)
        lp, lm, g, _ = _oracle_pair(ocfg, params, ids, seed)
        gp = [to_dev(p, torch) for p in params]
        ctx = zo.Context(cfg, gp, B, S)
        out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=seed, eps=EPS, lr=0.0).cpu().numpy()
        ctx.close()
        assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm)
        assert out[2] == orc.projected_grad(np.float32(out[0]), np.float32(out[1]), np.float32(EPS))
        dg.append(float(out[2]) - float(g))
        gs.append(float(g))
    dg, gs = np.array(dg), np.array(gs)
    rel = np.abs(dg) / np.abs(gs)
    print("bf16 A%d: |g| median %.3f; delta g mean %+.4f median |.| %.4f max %.4f; relative median %.4f max %.4f"
          % (a_bits, np.median(np.abs(gs)), dg.mean(), np.median(np.abs(dg)), np.abs(dg).max(), np.median(rel), rel.max()))
    assert np.median(np.abs(dg)) <= 0.15 and np.abs(dg).max() <= 0.6
    assert abs(dg.mean()) <= 0.15                     # no systematic shift
