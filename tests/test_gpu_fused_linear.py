"""GPU parity of the fused small-M form of the fake-quantized linear (tiles of Q(W +- eps u) of Eq. 2
built inside the GEMM kernel) against the oracle: the built tiles bit-exactly (an identity activation
matrix reads them out), layer outputs within 1e-2 relative (bf16 operands), the model forward through
that route against the oracle and against the quantize-once route."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev, rel_l2

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits,g", [(4, 64), (2, 64), (4, 128), (8, 32), (3, 16), (4, 8), (0, 0)])
def test_fused_tiles_bit_exact(bits, g):
    """X = identity (K = M = 128): Y[m][n] is exactly w^[n][m], for both branches."""
    torch, zo = gpu()
    N, K = 48, 128
    W = synth.weights((N, K), 61)
    eye = torch.eye(K, dtype=torch.bfloat16, device="cuda")
    eps = np.float32(1e-3)
    Yp, Ym = zo.zo_linear_fakequant_fused(eye, eye, to_dev(W, torch), None, bits, g, seed=7, tensor_id=3, eps=float(eps), relayout=True)
    for Y, e in ((Yp, eps), (Ym, -eps)):
        ref = orc.fakequant_weight(W, bits, g, 7, 3, np.float32(e), round_bf16=True, want_codes=False)["what"]
        assert np.array_equal(Y.float().cpu().numpy().T, ref)
    # single-branch call, fp32 output, eps = 0 (no stream drawn)
    Y0, none = zo.zo_linear_fakequant_fused(eye, None, to_dev(W, torch), None, bits, g, seed=7, tensor_id=3, eps=0.0, out_f32=True)
    assert none is None
    ref = orc.fakequant_weight(W, bits, g, 7, 3, np.float32(0), round_bf16=True, want_codes=False)["what"]
    assert np.array_equal(Y0.cpu().numpy().T, ref)


@pytest.mark.parametrize("M,N,K,bits,g", [(8, 256, 256, 4, 64), (1, 16, 64, 4, 64), (17, 80, 448, 2, 64), (100, 272, 1024, 4, 128),
                                          (128, 4096, 512, 4, 64), (33, 96, 4096, 4, 64), (128, 64, 11008, 4, 64),
                                          (60, 160, 992, 8, 32), (128, 512, 256, 0, 0)])
@pytest.mark.parametrize("out_f32,relayout", [(False, False), (True, False), (True, True)])
def test_fused_linear_vs_oracle(M, N, K, bits, g, out_f32, relayout):
    """Different activations per branch, bias, ragged M, many K slabs per wave and fewer slabs than waves."""
    torch, zo = gpu()
    Xp = orc.bf16_round(synth.activations((M, K), 62))
    Xm = orc.bf16_round(synth.activations((M, K), 63))
    W = synth.weights((N, K), 64)
    bias = synth.weights((N,), 65)
    eps = np.float32(1e-3)
    Yp, Ym = zo.zo_linear_fakequant_fused(to_dev(Xp, torch, torch.bfloat16), to_dev(Xm, torch, torch.bfloat16), to_dev(W, torch),
                                          to_dev(bias, torch), bits, g, seed=5, tensor_id=9, eps=float(eps), out_f32=out_f32,
                                          relayout=relayout)
    if relayout:                                    # the copy changes the order of the loads, not one bit of the result
        Yp2, Ym2 = zo.zo_linear_fakequant_fused(to_dev(Xp, torch, torch.bfloat16), to_dev(Xm, torch, torch.bfloat16), to_dev(W, torch),
                                                to_dev(bias, torch), bits, g, seed=5, tensor_id=9, eps=float(eps), out_f32=out_f32)
        assert torch.equal(Yp, Yp2) and torch.equal(Ym, Ym2)
    for Y, X, e in ((Yp, Xp, eps), (Ym, Xm, -eps)):
        what = orc.fakequant_weight(W, bits, g, 5, 9, np.float32(e), round_bf16=True, want_codes=False)["what"]
        ref = orc.linear(X, what, bias)
        got = Y.float().cpu().numpy()
        assert rel_l2(got, ref) < (1e-5 if out_f32 else 1e-2)
        # fp32 accumulation of K bf16 x bf16 products (+ one bf16 rounding of the result)
        mag = np.abs(X.astype(np.float64)) @ np.abs(what.astype(np.float64)).T + np.abs(bias)
        assert np.all(np.abs(got - ref) <= 2.0 ** -20 * mag + (2.0 ** -8 * np.abs(ref) if not out_f32 else 0.0) + 1e-30)


def test_fused_linear_matches_two_pass():
    """Same weights, same activations: the two routes differ only in the order of the fp32 accumulation."""
    torch, zo = gpu()
    M, N, K = 64, 384, 2048
    X = orc.bf16_round(synth.activations((M, K), 66))
    W = synth.weights((N, K), 67)
    xd, wd = to_dev(X, torch, torch.bfloat16), to_dev(W, torch)
    Yf, _ = zo.zo_linear_fakequant_fused(xd, None, wd, None, 4, 64, seed=2, tensor_id=1, eps=1e-3, out_f32=False)
    Yt = zo.zo_linear_fakequant(xd, wd, None, 4, 64, 16, 0, seed=2, tensor_id=1, eps_signed=1e-3)
    a, b = Yf.float().cpu().numpy(), Yt.float().cpu().numpy()
    assert np.mean(a != b) < 0.02                               # bf16 roundings that fall on different sides
    assert np.all(np.abs(a - b) <= 2.0 ** -7 * np.abs(b) + 1e-6)


def test_fused_rejects_unsupported_shapes():
    torch, zo = gpu()
    W = torch.zeros((16, 64), dtype=torch.float32, device="cuda")
    X = torch.zeros((129, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(zo.ZoError) as e:
        zo.zo_linear_fakequant_fused(X, None, W, None, 4, 64)            # M > 128
    assert e.value.status == 2
    with pytest.raises(zo.ZoError):
        zo.zo_linear_fakequant_fused(X[:8], None, W, None, 4, 0)         # per-channel groups
    with pytest.raises(zo.ZoError):
        zo.zo_linear_fakequant_fused(X[:8], None, W[:8], None, 4, 64)    # N not a multiple of 16
    with pytest.raises(zo.ZoError):
        zo.zo_linear_fakequant_fused(X[:8, :48].contiguous(), None, W[:, :48].contiguous(), None, 4, 16)   # K % 32


def _model(zo, arch, act_bits, no_fused, B, S, kw):
    return zo.make_config(arch, act_dtype=zo.ACT_BF16, a_bits=act_bits, no_fused=no_fused, **kw)


@pytest.mark.parametrize("arch,a_bits", [("llama", 16), ("llama", 8), ("opt", 8)])
def test_model_step_through_fused_route(arch, a_bits):
    """B*S = 96 tokens: every quantized linear and the lm_head take the fused kernel.  Losses against the oracle
    (1e-3 relative) and against the quantize-once route; the update is the same function of the losses."""
    torch, zo = gpu()
    kw = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=256, vocab=512, max_seq=48, w_bits=4, w_group=64)
    B, S = 2, 48                                    # 96 tokens: the activations go through the fragment-ordered copy
    oarch = orc.ARCH_LLAMA if arch == "llama" else orc.ARCH_OPT
    zarch = zo.ARCH_LLAMA if arch == "llama" else zo.ARCH_OPT
    ocfg = orc.Config(oarch, act_dtype=1, a_bits=a_bits, **kw)
    params = synth.model_params(orc.param_shapes(ocfg), 71)
    ids = synth.token_ids(B, S, kw["vocab"], 72)
    lp, lm, g = orc.zo_step(ocfg, [p.copy() for p in params], 13, 1e-3, 1e-4, ids=ids)
    outs = []
    for no_fused in (0, 1):
        gp = [to_dev(p, torch) for p in params]
        ctx = zo.Context(_model(zo, zarch, a_bits, no_fused, B, S, kw), gp, B, S)
        ctx.zo_profile_begin()
        out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=13, eps=1e-3, lr=1e-4).cpu().numpy().copy()
        prof = ctx.zo_profile_end()
        assert ctx.zo_debug_routes() & ~zo.ROUTE_GEMM_SPLIT_K == (0 if no_fused else zo.ROUTE_FUSED_SMALL_M)
        n_gemm = 4 * kw["n_layers"] + 1                         # GEMM launches of a forward pair (q/k/v and gate/up batched)
        # one fused launch per weight tensor, two tensors of one shape that feed on the same input in one launch: per layer
        # q + k, v, o, gate + up (Llama) or fc1 (OPT), down / fc2; and the lm_head
        n_lin = 5 * kw["n_layers"] + 1
        if no_fused:
            assert prof["fused_linear"][1] == 0 and prof["gemm"][1] == n_gemm
        else:
            assert prof["gemm"][1] == 0 and prof["fused_linear"][1] == n_lin
        outs.append(out)
        assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm)
        # g is exactly the oracle's function of the two device losses
        assert out[2] == np.float32(orc.projected_grad(out[0], out[1], 1e-3))
        ctx.close()
    assert abs(outs[0][0] - outs[1][0]) <= 2e-4 * abs(lp) and abs(outs[0][1] - outs[1][1]) <= 2e-4 * abs(lm)
