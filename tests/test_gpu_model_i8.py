"""zo_config.mma = ZO_MMA_INT8 through whole forwards and steps: every quantized linear of a forward that quantizes once
contracts its integer codes (signed-byte operands, int8 matrix instructions, steps and zero points in fp32) -- against the
oracle's model with the same switch (operands not rounded: Background/Quantization's X_INT contracted exactly).  Losses to
the tolerances of the bf16 route (1e-4 in fp32 storage, 1e-3 in bf16 storage), g exactly the quotient of the device's
losses, updated masters bit-exact given the device's coefficient."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu

EPS = 1e-3


def _step(arch, act_dtype, w_group, a_bits, w_bits=4, B=4, S=64, lr=1e-3):
    torch, zo = gpu()
    base = dict(n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=512, max_seq=S, w_bits=w_bits, w_group=w_group, a_bits=a_bits)
    ocfg = orc.Config(arch, act_dtype=act_dtype, mma=1, **base)
    cfg = zo.make_config(arch, act_dtype=act_dtype, mma=zo.MMA_INT8, **base)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 2300)
    ids = synth.token_ids(B, S, base["vocab"], 2301)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=3, eps=EPS, lr=lr).cpu().numpy()
    routes = ctx.zo_debug_routes()
    lp = orc.forward(ocfg, params, ids=ids, seed=3, eps_signed=np.float32(EPS))
    lm = orc.forward(ocfg, params, ids=ids, seed=3, eps_signed=np.float32(-EPS))
    tol = 1e-4 if act_dtype == 0 else 1e-3
    print("gpu L+ %.6f L- %.6f | oracle L+ %.6f L- %.6f | routes 0x%x" % (out[0], out[1], lp, lm, routes))
    assert routes & zo.ROUTE_INT8_MMA
    assert abs(out[0] - lp) <= tol * abs(lp) and abs(out[1] - lm) <= tol * abs(lm)
    assert out[2] == orc.projected_grad(np.float32(out[0]), np.float32(out[1]), np.float32(EPS))
    assert out[3] == orc.coeff(np.float32(lr), out[2])
    for i in (0, 2, len(shapes) - 1):
        assert np.array_equal(gp[i].cpu().numpy(), orc.update(params[i].copy(), 3, i, np.float32(out[3])))
    ctx.close()
    return out, (lp, lm)


@pytest.mark.parametrize("arch", [1, 2])
@pytest.mark.parametrize("act_dtype", [0, 1])
def test_step_on_integer_codes_groups_of_64(arch, act_dtype):
    _step(arch, act_dtype, 64, 8)


@pytest.mark.parametrize("w_group,a_bits", [(0, 8), (128, 4), (0, 4)])
def test_step_on_integer_codes_other_settings(w_group, a_bits):
    """per channel (no rescale inside the loop; the W4A4 rows of the appendix's quantization settings), a step per 128."""
    _step(1, 1, w_group, a_bits)


@pytest.mark.parametrize("w_group", [0, 64])
def test_step_on_integer_codes_with_the_swiglu_epilogue(w_group):
    """bf16 storage: the integer GEMM applies SwiGLU (gate | up rows interleaved) in its epilogue, like the bf16 one."""
    torch, zo = gpu()
    B, S = 2, 128
    base = dict(n_layers=2, d_model=256, n_heads=2, d_ffn=512, vocab=512, max_seq=S, w_bits=4, w_group=w_group, a_bits=8)
    ocfg = orc.Config(1, act_dtype=1, mma=1, **base)
    cfg = zo.make_config(1, act_dtype=1, mma=zo.MMA_INT8, **base)
    params = synth.model_params(orc.param_shapes(ocfg), 2340)
    ids = synth.token_ids(B, S, 512, 2341)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=9, eps=EPS, lr=1e-3).cpu().numpy()
    routes = ctx.zo_debug_routes()
    assert routes & zo.ROUTE_INT8_MMA and routes & zo.ROUTE_SWIGLU_IN_GEMM, hex(routes)
    lp = orc.forward(ocfg, params, ids=ids, seed=9, eps_signed=np.float32(EPS))
    lm = orc.forward(ocfg, params, ids=ids, seed=9, eps_signed=np.float32(-EPS))
    print("gpu L+ %.6f L- %.6f | oracle L+ %.6f L- %.6f" % (out[0], out[1], lp, lm))
    assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm)
    # the same forward with the stand-alone kernels (no_fused = 1 keeps the integer route but switches the epilogues off)
    cfg2 = zo.make_config(1, act_dtype=1, mma=zo.MMA_INT8, no_fused=1, **base)
    gp2 = [to_dev(p, torch) for p in params]
    ctx2 = zo.Context(cfg2, gp2, B, S)
    out2 = ctx2.zo_step(to_dev(ids, torch), None, B, S, seed=9, eps=EPS, lr=1e-3).cpu().numpy()
    r2 = ctx2.zo_debug_routes()
    assert r2 & zo.ROUTE_INT8_MMA and not r2 & (zo.ROUTE_ROPE_IN_GEMM | zo.ROUTE_SWIGLU_IN_GEMM)
    assert abs(out2[0] - out[0]) <= 2e-4 * abs(out[0]) and abs(out2[1] - out[1]) <= 2e-4 * abs(out[1]), (out, out2)
    ctx.close()
    ctx2.close()


def test_integer_route_differs_from_the_bf16_route_by_the_operand_rounding_only():
    """bf16 storage: the two contractions see the same codes; the integer one does not round the de-quantized operands to
    bf16, so the losses differ by a few 1e-4 relative -- and each agrees with its own oracle."""
    torch, zo = gpu()
    out_i, (lp_i, _) = _step(1, 1, 64, 8)
    base = dict(n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=512, max_seq=64, w_bits=4, w_group=64, a_bits=8)
    ocfg = orc.Config(1, act_dtype=1, mma=0, **base)
    params = synth.model_params(orc.param_shapes(ocfg), 2300)
    ids = synth.token_ids(4, 64, 512, 2301)
    lp_b = orc.forward(ocfg, params, ids=ids, seed=3, eps_signed=np.float32(EPS))
    assert lp_b != lp_i and abs(lp_b - lp_i) <= 2e-3 * abs(lp_b)


def test_single_linear_configuration_on_integer_codes():
    """The single-linear regression configuration (256 -> 256, W4 group 64, A8, 8 rows) with fp32 storage, which quantizes once."""
    torch, zo = gpu()
    base = dict(d_model=256, d_ffn=256, w_bits=4, w_group=64, a_bits=8)
    ocfg = orc.Config(orc.ARCH_LINEAR, act_dtype=0, mma=1, **base)
    cfg = zo.make_config(0, act_dtype=0, mma=zo.MMA_INT8, **base)
    W = synth.weights((256, 256), 2310)
    X = synth.activations((8, 256), 2311)
    T = synth.activations((8, 256), 2312)
    gp = [to_dev(W, torch)]
    ctx = zo.Context(cfg, gp, 8, 1)
    out = ctx.zo_step(to_dev(X, torch), to_dev(T, torch), 8, 1, seed=0, eps=EPS, lr=1e-4).cpu().numpy()
    assert ctx.zo_debug_routes() & zo.ROUTE_INT8_MMA
    lp = orc.forward(ocfg, [W], x=X, target=T, seed=0, eps_signed=np.float32(EPS))
    lm = orc.forward(ocfg, [W], x=X, target=T, seed=0, eps_signed=np.float32(-EPS))
    assert abs(out[0] - lp) <= 1e-5 * abs(lp) and abs(out[1] - lm) <= 1e-5 * abs(lm), (out, lp, lm)
    assert np.array_equal(gp[0].cpu().numpy(), orc.update(W.copy(), 0, 0, np.float32(out[3])))
    ctx.close()


def test_configurations_the_integer_route_cannot_express_are_refused():
    torch, zo = gpu()
    ok = dict(n_layers=1, d_model=256, n_heads=4, d_ffn=512, vocab=128, max_seq=8, w_bits=4, w_group=64, a_bits=8)
    for bad in (dict(a_bits=16), dict(w_bits=8), dict(w_group=32), dict(d_ffn=384), dict(d_model=128, n_heads=2)):
        cfg = zo.make_config(1, act_dtype=1, mma=zo.MMA_INT8, **{**ok, **bad})
        assert zo.zo_workspace_bytes(cfg, 1, 8) == 0, bad


def test_operands_that_do_not_fit_a_byte_poison_the_losses():
    """A weight row far from zero compared with its own range has |code - zero point| in the thousands: the integer route cannot
    represent it, the forward says so through NaN losses (and the next forward starts from a clear flag)."""
    torch, zo = gpu()
    base = dict(n_layers=1, d_model=256, n_heads=4, d_ffn=512, vocab=512, max_seq=64, w_bits=4, w_group=64, a_bits=8)
    cfg = zo.make_config(1, act_dtype=1, mma=zo.MMA_INT8, **base)
    shapes = orc.param_shapes(orc.Config(1, act_dtype=1, **base))
    params = synth.model_params(shapes, 2320)
    good = [to_dev(p, torch) for p in params]
    bad = [to_dev(p, torch) for p in params]
    flat = bad[2].view(-1)
    flat[5 * 256:6 * 256] = 1.0 + 1e-3 * flat[5 * 256:6 * 256]              # row 5 of wq
    ids = to_dev(synth.token_ids(4, 64, 512, 2321), torch)
    ctx = zo.Context(cfg, bad, 4, 64)
    out = ctx.zo_forward_quant(ids, None, 4, 64, seed=1, eps_signed=0.0).cpu().numpy()
    assert np.isnan(out[0])
    ctx.close()
    ctx = zo.Context(cfg, good, 4, 64)
    out = ctx.zo_forward_quant(ids, None, 4, 64, seed=1, eps_signed=0.0).cpu().numpy()
    assert np.isfinite(out[0])
    ctx.close()


def test_integer_route_with_binary16_masters():
    """Masters kept in IEEE binary16 (per-channel steps, so the row quantizer's register-held form reads them)."""
    torch, zo = gpu()
    B, S = 4, 64
    base = dict(n_layers=1, d_model=256, n_heads=4, d_ffn=512, vocab=512, max_seq=S, w_bits=4, w_group=0, a_bits=8)
    ocfg = orc.Config(1, act_dtype=1, mma=1, **base)
    cfg = zo.make_config(1, act_dtype=1, mma=zo.MMA_INT8, master_dtype=zo.MASTER_F16, **base)
    params = [p.astype(np.float16) for p in synth.model_params(orc.param_shapes(ocfg), 2330)]
    ids = synth.token_ids(B, S, 512, 2331)
    lp, lm, g = orc.zo_step(ocfg, [p.copy() for p in params], 5, EPS, 1e-3, ids=ids, stochastic=False)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=5, eps=EPS, lr=1e-3).cpu().numpy()
    assert ctx.zo_debug_routes() & zo.ROUTE_INT8_MMA
    assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm), (out, lp, lm)
    want = orc.update(params[2].copy(), 5, 2, np.float32(out[3]), False)
    assert np.array_equal(gp[2].cpu().numpy().view(np.uint16), want.view(np.uint16))
    ctx.close()
