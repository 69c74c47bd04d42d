"""GPU parity of the q-direction step (Eq. 2 with q > 1, Eq. 3), the one-pass multi-direction update and the replay
of a run from its (seeds, coefficients) log, against the oracle.  Losses 1e-3 relative (1e-4 with fp32 storage);
g_i and the coefficients are exactly the oracle's functions of the device losses; the updated masters are bit-exact
given those coefficients."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


def _check_outputs(out, eps, lrs, q):
    """Row i of out = {L+, L-, g_i, c_model, c_smooth, c_clip}: g and c as the oracle computes them from the losses."""
    for i in range(q):
        g = orc.projected_grad(out[i, 0], out[i, 1], np.float32(eps))
        assert out[i, 2] == g
        for j, lr in enumerate(lrs):
            assert out[i, 3 + j] == orc.coeff(np.float32(np.float32(lr) / np.float32(q)), g)


@pytest.mark.parametrize("N,K,q", [(24, 72, 3), (96, 160, 1), (200, 328, 4), (64, 64, 16)])
def test_linear_layer_multi_step(N, K, q):
    """Tensors smaller than, equal to and larger than the update kernel's 4096-element blocks, with ragged ends."""
    torch, zo = gpu()
    kw = dict(d_model=K, d_ffn=N, w_bits=4, w_group=8, a_bits=8)
    ocfg = orc.Config(orc.ARCH_LINEAR, act_dtype=0, **kw)
    cfg = zo.make_config(zo.ARCH_LINEAR, act_dtype=zo.ACT_FP32, **kw)
    M = 8
    W = synth.weights((N, K), 81)
    X, T = synth.activations((M, K), 82), synth.activations((M, N), 83)
    seeds = [1000 + 7 * i for i in range(q)]
    eps, lr = 1e-3, 1e-2
    ref_w = [W.copy()]
    ref = orc.zo_step_multi(ocfg, ref_w, seeds, eps, lr, x=X, target=T)
    gw = [to_dev(W, torch)]
    ctx = zo.Context(cfg, gw, M, 1)
    out = ctx.zo_step_multi(to_dev(X, torch), to_dev(T, torch), M, 1, seeds, eps, lr).cpu().numpy()
    for i, (lp, lm, g) in enumerate(ref):
        assert abs(out[i, 0] - lp) <= 1e-4 * abs(lp) and abs(out[i, 1] - lm) <= 1e-4 * abs(lm)
    _check_outputs(out, eps, (lr, lr, lr), q)
    # masters: the oracle's update applied with the device's own coefficients, in seed order, is bit-exact
    w = W.copy()
    for s, row in zip(seeds, out):
        orc.update(w, s, 0, np.float32(row[3]))
    assert np.array_equal(gw[0].cpu().numpy(), w)
    ctx.close()


@pytest.mark.parametrize("arch,learn", [("llama", 0), ("opt", 1)])
def test_decoder_multi_step(arch, learn):
    torch, zo = gpu()
    kw = dict(n_layers=2, d_model=64, n_heads=4, d_ffn=128, vocab=256, max_seq=24, w_bits=4, w_group=32, a_bits=8,
              learn_clip=learn, learn_smooth=learn)
    B, S, q = 2, 24, 3
    oarch, zarch = (orc.ARCH_LLAMA, zo.ARCH_LLAMA) if arch == "llama" else (orc.ARCH_OPT, zo.ARCH_OPT)
    ocfg = orc.Config(oarch, act_dtype=0, **kw)
    cfg = zo.make_config(zarch, act_dtype=zo.ACT_FP32, **kw)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 84)
    if learn:
        orc.init_learned_params(ocfg, params)
    ids = synth.token_ids(B, S, kw["vocab"], 85)
    seeds = [11, 12, 13]
    eps, lrs = 1e-3, (1e-3, 5e-4, 2e-4)
    ref_p = [p.copy() for p in params]
    ref = orc.zo_step_multi(ocfg, ref_p, seeds, eps, lrs[0], ids=ids, lr_smooth=lrs[1], lr_clip=lrs[2])
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    out = ctx.zo_step_multi(to_dev(ids, torch), None, B, S, seeds, eps, *lrs).cpu().numpy()
    for i, (lp, lm, g) in enumerate(ref):
        assert abs(out[i, 0] - lp) <= 1e-3 * abs(lp) and abs(out[i, 1] - lm) <= 1e-3 * abs(lm)
    _check_outputs(out, eps, lrs, q)
    groups = orc.param_groups(ocfg)
    for t, (p0, g) in enumerate(zip(params, groups)):
        w = p0.copy()
        for s, row in zip(seeds, out):
            orc.update(w, s, t, np.float32(row[3 + g]))
        assert np.array_equal(gp[t].cpu().numpy(), w), shapes[t][0]
    ctx.close()


def test_q1_is_zo_step_groups():
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=64, n_heads=2, d_ffn=128, vocab=128, max_seq=16, w_bits=4, w_group=64, a_bits=16)
    cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=zo.ACT_BF16, **kw)
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=1, **kw)
    params = synth.model_params(orc.param_shapes(ocfg), 86)
    ids = to_dev(synth.token_ids(2, 16, 128, 87), torch)
    a = [to_dev(p, torch) for p in params]
    b = [to_dev(p, torch) for p in params]
    ca, cb = zo.Context(cfg, a, 2, 16), zo.Context(cfg, b, 2, 16)
    oa = ca.zo_step_groups(ids, None, 2, 16, 5, 1e-3, 1e-3, 2e-3, 3e-3).cpu().numpy()
    ob = cb.zo_step_multi(ids, None, 2, 16, [5], 1e-3, 1e-3, 2e-3, 3e-3).cpu().numpy()
    assert np.array_equal(oa, ob[0])
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    ca.close(); cb.close()


def test_replay_from_log_and_argument_checks():
    """Four 2-direction steps under the linear-decay schedule; replaying the (seeds, coefficients) log on the initial
    masters -- from host coefficients and from the device rows -- reproduces every tensor bit for bit."""
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=64, n_heads=2, d_ffn=128, vocab=128, max_seq=16, w_bits=4, w_group=64, a_bits=8)
    cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=zo.ACT_BF16, **kw)
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=1, **kw)
    params = synth.model_params(orc.param_shapes(ocfg), 88)
    ids = to_dev(synth.token_ids(2, 16, 128, 89), torch)
    run = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, run, 2, 16)
    log = []
    T = 4
    for t in range(T):
        lr = zo.zo_lr_linear_decay(1e-2, t, T)
        seeds = [2 * t, 2 * t + 1]
        out = ctx.zo_step_multi(ids, None, 2, 16, seeds, 1e-3, lr).clone()
        log.append((seeds, out))
    assert not torch.equal(run[1], to_dev(params[1], torch))
    for mode in ("host", "dev"):
        rep = [to_dev(p, torch) for p in params]
        c2 = zo.Context(cfg, rep, 2, 16)
        for seeds, out in log:
            if mode == "host":
                c2.zo_update_multi(seeds, coeff_host=out[:, 3:6].cpu().tolist())
            else:
                c2.zo_update_multi(seeds, coeff_dev=out)
        for x, y in zip(run, rep):
            assert torch.equal(x, y)
        c2.close()
    for bad in ([], list(range(17))):
        with pytest.raises(zo.ZoError) as e:
            ctx.zo_step_multi(ids, None, 2, 16, bad, 1e-3, 1e-3)
        assert e.value.status == 1
    ctx.close()
