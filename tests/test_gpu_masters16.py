"""GPU parity of master weights kept in IEEE binary16 (the 2 bytes per parameter of the paper's memory table):
the update (fp32 fma, one rounding, nearest-even or stochastic) bit-exactly, whole steps against the oracle through
both linear routes, and q-direction steps with a single rounding."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [5, 8, 4099, 100003])
@pytest.mark.parametrize("stochastic", [False, True])
def test_update_tensor_f16_bit_exact(n, stochastic):
    torch, zo = gpu()
    w0 = synth.weights((n,), 91).astype(np.float16)
    w0[: min(n, 3)] = [0.0, -0.0, 6e-8][: min(n, 3)]                  # zeros and a binary16 subnormal
    for c in (np.float32(3e-3), np.float32(1e-6), np.float32(0.0)):
        ref = orc.update(w0.copy(), 17, 6, c, stochastic)
        w = to_dev(w0, torch)
        zo.zo_update_tensor_f16(w, 17, 6, coeff_host=float(c), stochastic=stochastic)
        assert np.array_equal(w.cpu().numpy().view(np.uint16), ref.view(np.uint16))
        w = to_dev(w0, torch)
        zo.zo_update_tensor_f16(w, 17, 6, coeff_dev=to_dev(np.array([c], np.float32), torch), stochastic=stochastic)
        assert np.array_equal(w.cpu().numpy().view(np.uint16), ref.view(np.uint16))


def test_stochastic_rounding_keeps_small_steps_on_the_gpu():
    torch, zo = gpu()
    n = 1 << 20
    w = torch.ones(n, dtype=torch.float16, device="cuda")
    zo.zo_update_tensor_f16(w, 3, 0, coeff_host=1e-5, stochastic=False)
    assert bool((w == 1).all())                                       # nearest-even: every step lost
    zo.zo_update_tensor_f16(w, 3, 0, coeff_host=1e-5, stochastic=True)
    step = w.double().cpu().numpy() - 1.0
    z = orc.normal(3, 0, n).astype(np.float64)
    assert abs(np.sum(step * z) + 1e-5 * np.sum(z * z)) < 5 * np.sqrt(np.sum(2.0 ** -10 * 1e-5 * np.abs(z) ** 3))


@pytest.mark.parametrize("arch", ["llama", "opt"])
@pytest.mark.parametrize("act_dtype,no_fused", [(0, 0), (1, 0), (1, 1)])
@pytest.mark.parametrize("stochastic", [0, 1])
def test_step_with_f16_masters(arch, act_dtype, no_fused, stochastic):
    """fp32 storage (quantize-once route), bf16 storage through the fused small-M kernel and through the quantize-once
    route.  Losses against the oracle; masters bit-exact given the device's own coefficient."""
    torch, zo = gpu()
    kw = dict(n_layers=2, d_model=64, n_heads=4, d_ffn=128, vocab=256, max_seq=24, w_bits=4, w_group=32, a_bits=8)
    B, S = 2, 24
    oarch, zarch = (orc.ARCH_LLAMA, zo.ARCH_LLAMA) if arch == "llama" else (orc.ARCH_OPT, zo.ARCH_OPT)
    ocfg = orc.Config(oarch, act_dtype=act_dtype, **kw)
    cfg = zo.make_config(zarch, act_dtype=act_dtype, no_fused=no_fused, master_dtype=zo.MASTER_F16, master_round=stochastic, **kw)
    params = [p.astype(np.float16) for p in synth.model_params(orc.param_shapes(ocfg), 92)]
    ids = synth.token_ids(B, S, kw["vocab"], 93)
    ref_p = [p.copy() for p in params]
    lp, lm, g = orc.zo_step(ocfg, ref_p, 21, 1e-3, 2e-3, ids=ids, stochastic=bool(stochastic))
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=21, eps=1e-3, lr=2e-3).cpu().numpy()
    tol = 1e-3 if act_dtype else 1e-4
    assert abs(out[0] - lp) <= tol * abs(lp) and abs(out[1] - lm) <= tol * abs(lm)
    assert out[2] == orc.projected_grad(out[0], out[1], np.float32(1e-3)) and out[3] == orc.coeff(np.float32(2e-3), out[2])
    for t, p0 in enumerate(params):
        want = orc.update(p0.copy(), 21, t, np.float32(out[3]), bool(stochastic))
        assert np.array_equal(gp[t].cpu().numpy().view(np.uint16), want.view(np.uint16)), t
    assert any(not np.array_equal(gp[t].cpu().numpy(), params[t]) for t in range(len(params)))
    ctx.close()


def test_multi_direction_step_with_f16_masters():
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=64, n_heads=2, d_ffn=128, vocab=128, max_seq=16, w_bits=4, w_group=64, a_bits=16)
    cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=zo.ACT_FP32, master_dtype=zo.MASTER_F16, master_round=1, **kw)
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=0, **kw)
    params = [p.astype(np.float16) for p in synth.model_params(orc.param_shapes(ocfg), 94)]
    ids = synth.token_ids(2, 16, 128, 95)
    seeds = [7, 8, 9]
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, 2, 16)
    out = ctx.zo_step_multi(to_dev(ids, torch), None, 2, 16, seeds, 1e-3, 3e-3).cpu().numpy()
    ref = orc.zo_step_multi(ocfg, [p.copy() for p in params], seeds, 1e-3, 3e-3, ids=ids, stochastic=True)
    for i, (lp, lm, g) in enumerate(ref):
        assert abs(out[i, 0] - lp) <= 1e-4 * abs(lp) and abs(out[i, 1] - lm) <= 1e-4 * abs(lm)
    for t, p0 in enumerate(params):
        want = orc.update_multi(p0.copy(), seeds, t, [np.float32(r[3]) for r in out], True)
        assert np.array_equal(gp[t].cpu().numpy().view(np.uint16), want.view(np.uint16)), t
    ctx.close()
