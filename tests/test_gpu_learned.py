"""GPU parity of the adaptive weight quantizer (Eq. 5) and channel-wise smoothing (Eq. 4) as ZO-trained
tensors: the weight kernel is bit-exact against the oracle (integer codes, de-quantized values), the
bias term of Eq. 4 agrees to fp32 accumulation noise, the initial parameters equal the oracle's, and
whole steps with three learning-rate groups match the oracle's step (losses 1e-3; every tensor moved
by exactly its group's coefficient times u)."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,K,bits,group", [(24, 256, 4, 64), (16, 384, 2, 128), (40, 512, 4, 0), (8, 64, 8, 8)])
@pytest.mark.parametrize("with_scale", [False, True])
@pytest.mark.parametrize("out_dtype", [0, 1])
def test_learned_weight_quantizer_is_bit_exact(N, K, bits, group, with_scale, out_dtype):
    torch, zo = gpu()
    rng = synth.rng(701)
    W = synth.weights((N, K), 702)
    scale = (1.0 + rng.uniform(-0.4, 0.6, K)).astype(np.float32) if with_scale else None
    step, zp, alpha, beta = orc.init_learned(W, bits, group, scale)
    G = step.shape[1]
    # move the parameters off their initial values the way a perturbation would
    step = (step * (1.0 + 0.2 * rng.standard_normal((N, G)))).astype(np.float32)
    step[0, 0] = -1e-3                                   # below the floor
    zp = (zp + 0.8 * rng.standard_normal((N, G))).astype(np.float32)
    alpha = (alpha + 0.15 * rng.standard_normal((N, G))).astype(np.float32)
    beta = (beta + 0.15 * rng.standard_normal((N, G))).astype(np.float32)
    eps = np.float32(1e-3)
    ref = orc.fakequant_weight_learned(W, bits, group, step, zp, alpha, beta, scale=scale, seed=5, tensor_id=3, eps_signed=eps,
                                       round_bf16=bool(out_dtype))
    d = lambda a: None if a is None else to_dev(a, torch)
    out = zo.zo_debug_quant_weight_learned(d(W), bits, group, d(step), d(zp), d(alpha), d(beta), scale=d(scale), seed=5, tensor_id=3,
                                           eps_signed=float(eps), out_dtype=out_dtype)
    assert np.array_equal(out["codes"].cpu().numpy().astype(np.int32), ref["codes"])
    assert np.array_equal(out["what"].float().cpu().numpy().view(np.uint32), ref["what"].view(np.uint32))


def test_smoothed_bias_term():
    torch, zo = gpu()
    N, K = 70, 640
    W = synth.weights((N, K), 703, scale=1.0)
    delta = synth.weights((K,), 704, scale=0.3)
    bias = synth.weights((N,), 705)
    eps = np.float32(-1e-3)
    wp = orc.perturb(W, 9, 4, eps)
    ref = bias.astype(np.float64) + wp.astype(np.float64) @ delta.astype(np.float64)
    got = zo.zo_debug_smooth_bias(to_dev(W, torch), to_dev(delta, torch), to_dev(bias, torch), seed=9, tensor_id=4,
                                  eps_signed=float(eps)).cpu().numpy()
    assert np.max(np.abs(got - ref)) <= 1e-5 * np.sqrt(K) * np.max(np.abs(ref))
    got0 = zo.zo_debug_smooth_bias(to_dev(W, torch), to_dev(delta, torch), None, seed=9, tensor_id=4, eps_signed=float(eps)).cpu().numpy()
    assert np.max(np.abs(got0 - (ref - bias))) <= 1e-5 * np.sqrt(K) * np.max(np.abs(ref))


def _setup(zo, torch, arch, act_dtype, B, S, **kw):
    base = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=256, vocab=512, max_seq=S, w_bits=4, w_group=64, a_bits=8)
    base.update(kw)
    ocfg = orc.Config(arch, act_dtype=act_dtype, **base)
    cfg = zo.make_config(arch, act_dtype=act_dtype, **base)
    shapes = orc.param_shapes(ocfg)
    assert zo.zo_num_params(cfg) == len(shapes)
    assert all(zo.zo_param_numel(cfg, i) == int(np.prod(sh)) for i, (_, sh, _) in enumerate(shapes))
    params = synth.model_params(shapes, 706)
    params = [p * (3.0 if (p.ndim == 2 and i < len(orc._base_param_shapes(ocfg))) else 1.0) for i, p in enumerate(params)]
    ids = synth.token_ids(B, S, base["vocab"], 707)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    return ocfg, params, ids, gp, ctx


@pytest.mark.parametrize("arch", [1, 2])
@pytest.mark.parametrize("flags", [dict(learn_clip=1), dict(learn_clip=1, learn_smooth=1)])
def test_initial_parameters_match_the_oracle(arch, flags):
    torch, zo = gpu()
    ocfg, params, ids, gp, ctx = _setup(zo, torch, arch, 0, 2, 16, **flags)
    ctx.zo_init_learned_params()
    orc.init_learned_params(ocfg, params)
    for i, (name, _, _) in enumerate(orc.param_shapes(ocfg)):
        assert np.array_equal(gp[i].cpu().numpy().reshape(params[i].shape), params[i]), name
    ctx.close()


@pytest.mark.parametrize("arch", [1, 2])
@pytest.mark.parametrize("act_dtype,a_bits,flags", [(0, 16, dict(learn_clip=1)), (0, 8, dict(learn_clip=1, learn_smooth=1)),
                                                   (1, 8, dict(learn_clip=1, learn_smooth=1)), (1, 4, dict(learn_clip=1))])
def test_step_with_learning_rate_groups(arch, act_dtype, a_bits, flags):
    torch, zo = gpu()
    B, S = 2, 24
    ocfg, params, ids, gp, ctx = _setup(zo, torch, arch, act_dtype, B, S, a_bits=a_bits, **flags)
    orc.init_learned_params(ocfg, params)
    rng = synth.rng(708)
    for i, (name, shape, _) in enumerate(orc.param_shapes(ocfg)):      # a non-trivial smoothing and clipping state
        if name.endswith(".sm_s"):
            params[i][...] = (1.0 + rng.uniform(-0.2, 0.4, shape)).astype(np.float32)
        if name.endswith(".sm_delta"):
            params[i][...] = (0.05 * rng.standard_normal(shape)).astype(np.float32)
        if name.endswith(".q_alpha"):
            params[i][...] = 0.04
        if name.endswith(".q_beta"):
            params[i][...] = 0.97
    if flags.get("learn_smooth"):                                        # step / zero point consistent with the smoothed weights
        index = {n: j for j, (n, _, _) in enumerate(orc.param_shapes(ocfg))}
        for name, shape, q in orc._base_param_shapes(ocfg):
            if q:
                st, z, _, _ = orc.init_learned(params[index[name]], 4, 64, params[index[orc.smooth_owner(name) + ".sm_s"]])
                params[index[name + ".q_step"]][...] = st
                params[index[name + ".q_zp"]][...] = z
    for t, p in zip(gp, params):
        t.copy_(torch.from_numpy(np.ascontiguousarray(p)).reshape(t.shape))
    idd = to_dev(ids, torch)
    tol = 3e-3 if act_dtype else 1e-3
    for eps in (0.0, 1e-3):
        loss = ctx.zo_forward_quant(idd, None, B, S, seed=6, eps_signed=eps).item()
        ref = orc.forward(ocfg, params, ids=ids, seed=6, eps_signed=eps)
        assert abs(loss - ref) <= tol * abs(ref), (eps, loss, ref)
    lrs = (1e-2, 3e-2, 5e-2)
    out = ctx.zo_step_groups(idd, None, B, S, 6, 1e-3, *lrs).cpu().numpy()
    before = [p.copy() for p in params]
    lp, lm, g = orc.zo_step(ocfg, params, 6, 1e-3, lrs[0], ids=ids, lr_smooth=lrs[1], lr_clip=lrs[2])
    assert abs(out[0] - lp) <= tol * abs(lp) and abs(out[1] - lm) <= tol * abs(lm)
    assert out[2] == orc.projected_grad(np.float32(out[0]), np.float32(out[1]), np.float32(1e-3))
    if act_dtype == 0 and a_bits == 16:
        assert abs(out[2] - g) <= 1e-3 * abs(g) + 5e-3
    groups = orc.param_groups(ocfg)
    for j in range(3):
        assert out[3 + j] == orc.coeff(np.float32(lrs[j]), np.float32(out[2]))
    for i, p0 in enumerate(before):
        want = orc.update(p0.copy(), 6, i, np.float32(out[3 + groups[i]]))
        assert np.array_equal(gp[i].cpu().numpy().reshape(p0.shape), want), i
    ctx.close()


def test_single_linear_with_learned_parameters():
    torch, zo = gpu()
    kw = dict(d_model=256, d_ffn=128, w_bits=4, w_group=64, a_bits=8, act_dtype=0, learn_clip=1, learn_smooth=1)
    ocfg = orc.Config(0, **kw)
    cfg = zo.make_config(0, **kw)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 709)
    orc.init_learned_params(ocfg, params)
    rng = synth.rng(710)
    params[5][...] = (1.0 + rng.uniform(-0.2, 0.4, 256)).astype(np.float32)       # s
    params[6][...] = (0.1 * rng.standard_normal(256)).astype(np.float32)          # delta
    x = synth.activations((8, 256), 711)
    target = synth.activations((8, 128), 712)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, 8, 1)
    out = ctx.zo_step_groups(to_dev(x, torch), to_dev(target, torch), 8, 1, 2, 1e-3, 1e-3, 1e-3, 1e-3).cpu().numpy()
    lp, lm, g = orc.zo_step(ocfg, params, 2, 1e-3, 1e-3, x=x, target=target)
    assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm)
    ctx.close()


def test_unsupported_combinations_are_refused():
    torch, zo = gpu()
    base = dict(n_layers=1, d_model=128, n_heads=4, d_ffn=256, vocab=64, max_seq=8, w_bits=4, w_group=64)
    for kw in (dict(a_bits=16, learn_clip=1, learn_smooth=1), dict(a_bits=8, learn_smooth=1), dict(a_bits=8, learn_clip=1, lightweight=1)):
        cfg = zo.make_config(1, act_dtype=0, **base, **kw)
        assert zo.zo_workspace_bytes(cfg, 1, 8) == 0


def test_learned_clipping_through_the_gemm_epilogues():
    """6 x 1024 tokens, 4 heads of 128, learned clipping (Eq. 5) without smoothing: the learned weight quantizer writes the
    q | k | v rows with the head blocks permuted and the gate / up rows interleaved, so the rotary embedding and SwiGLU
    run in the GEMM epilogues as they do with the dynamic quantizer.  Loss against the oracle and against the route with
    the stand-alone kernels; every parameter group moved by its own coefficient."""
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=512, n_heads=4, d_ffn=1024, vocab=256, max_seq=1024, w_bits=4, w_group=64, a_bits=8, learn_clip=1)
    B, S = 6, 1024
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=1, **kw)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 711)
    orc.init_learned_params(ocfg, params)
    for i, (name, shape, _) in enumerate(shapes):
        if name.endswith(".q_alpha"):
            params[i][...] = 0.04
        if name.endswith(".q_beta"):
            params[i][...] = 0.97
    ids = synth.token_ids(B, S, 256, 712)
    ref = orc.forward(ocfg, params, ids=ids, seed=8, eps_signed=1e-3)
    losses = []
    for no_fused in (0, 1):
        cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=1, no_fused=no_fused, **kw)
        gp = [to_dev(w, torch) for w in params]
        ctx = zo.Context(cfg, gp, B, S)
        idd = to_dev(ids, torch)
        losses.append(ctx.zo_forward_quant(idd, None, B, S, seed=8, eps_signed=1e-3).item())
        assert ctx.zo_debug_routes() & ~zo.ROUTE_GEMM_SPLIT_K == (0 if no_fused else zo.ROUTE_SWIGLU_IN_GEMM | zo.ROUTE_ROPE_IN_GEMM)
        assert abs(losses[-1] - ref) <= 3e-3 * abs(ref), (losses[-1], ref)
        if not no_fused:
            lrs = (1e-2, 3e-2, 5e-2)
            out = ctx.zo_step_groups(idd, None, B, S, 6, 1e-3, *lrs).cpu().numpy()
            groups = orc.param_groups(ocfg)
            for i in (0, 1, 2, len(params) - 1):
                want = orc.update(params[i].copy(), 6, i, np.float32(out[3 + groups[i]]))
                assert np.array_equal(gp[i].cpu().numpy().reshape(params[i].shape), want), i
        ctx.close()
    assert abs(losses[0] - losses[1]) <= 2e-4 * abs(ref)
