"""GPU parity of the quantized linear that contracts the integer codes with the int8 matrix instructions
(zo_linear_fakequant_mma, ZO_MMA_INT8): activation and weight operands bit-exact against the oracle's codes, the
rank-one zero-point term against its definition, and the layer output against the oracle's linear on UN-rounded
de-quantized operands (fp32 output: 1e-4 as in fp32 mode -- the result carries no operand rounding at all; bf16 output:
one storage rounding on top)."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,N,K,w_bits,group,a_bits,sym", [
    (8, 256, 256, 4, 64, 8, False),          # the single-linear configuration's widths
    (300, 520, 384, 4, 64, 8, False),        # ragged M and N, several tiles
    (257, 250, 512, 4, 128, 8, False),       # a step per 128
    (64, 100, 1024, 2, 256, 4, False),       # a step per two K tiles, 4-bit activations
    (130, 272, 512, 7, 512, 8, True),        # per channel (K = 512), symmetric activations
    (1, 16, 128, 3, 64, 6, False),
    (300, 520, 1152, 4, 0, 8, False),        # per channel: integer accumulation over all nine K tiles, ragged M and N
    (40, 96, 11008, 4, 0, 4, False),         # per channel over the widest row of the benchmark shapes, 4-bit activations
])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_int8_linear_vs_oracle(M, N, K, w_bits, group, a_bits, sym, dtype):
    torch, zo = gpu()
    X = synth.activations((M, K), 1301)
    X[M // 2] = np.abs(X[M // 2]) + 0.5                      # an all-positive row: zero point below zero
    if dtype == "bf16":
        X = orc.bf16_round(X)
    W = synth.weights((N, K), 1302)
    bias = synth.weights((N,), 1303)
    eps = np.float32(-1e-3)
    Xd = to_dev(X, torch, torch.bfloat16 if dtype == "bf16" else None)
    qa = orc.fakequant_act(X, a_bits, sym)
    qw = orc.fakequant_weight(W, w_bits, group, seed=21, tensor_id=4, eps_signed=eps)
    for out_f32 in (True, False):
        Y, parts = zo.zo_linear_fakequant_mma(Xd, to_dev(W, torch), w_bits, group, a_bits, 21, 4, float(eps), bias=to_dev(bias, torch),
                                              a_sym=sym, out_f32=out_f32, parts=True)
        off = 0 if sym else 1 << (a_bits - 1)
        assert np.array_equal(parts["x_codes"].cpu().numpy().astype(np.int32) + off, qa["codes"])
        assert np.array_equal(parts["x_step"].cpu().numpy().view(np.uint32), qa["step"].view(np.uint32))
        assert np.array_equal(parts["x_off"].cpu().numpy(), (off - qa["zp"]).astype(np.float32))
        gsz = group or K
        G = K // gsz
        wc = parts["w_codes"].cpu().numpy().astype(np.int32).reshape(N, G, gsz)
        assert np.array_equal(wc + qw["zp"][:, :, None], qw["codes"].reshape(N, G, gsz))
        rp = qw["step"].astype(np.float64) * wc.sum(-1)
        if G > 1:                                                         # (per channel there are no per-group parts: r is written directly)
            assert np.allclose(parts["w_rpart"].cpu().numpy(), rp, rtol=1e-6, atol=0)
        assert np.allclose(parts["w_r"].cpu().numpy(), rp.sum(-1), rtol=1e-5, atol=1e-6 * np.abs(rp).sum(-1).max())
        ref = orc.linear(qa["xhat"], qw["what"], bias)                    # un-rounded operands
        mag = np.abs(qa["xhat"].astype(np.float64)) @ np.abs(qw["what"].astype(np.float64)).T + np.abs(bias)
        got = Y.float().cpu().numpy()
        tol = 4e-6 * mag + (0.0 if out_f32 else 2.0 ** -8 * np.abs(ref))
        assert np.all(np.abs(got - ref) <= tol + 1e-30), (np.abs(got - ref) / mag).max()
        if out_f32:
            assert np.linalg.norm(got - ref) <= 1e-4 * np.linalg.norm(ref)


def test_int8_linear_flags_operands_that_do_not_fit_a_byte():
    torch, zo = gpu()
    M, N, K = 16, 32, 128
    X = to_dev(synth.activations((M, K), 1311), torch)
    W = synth.weights((N, K), 1312)
    W[5] = 1.0 + 1e-3 * W[5]                                  # a row far from zero compared with its range: |q - zp| ~ 1e4
    with pytest.raises(zo.ZoError) as e:
        zo.zo_linear_fakequant_mma(X, to_dev(W, torch), 4, 64, 8, 1, 0, 0.0)
    assert e.value.status == 5
    with pytest.raises(zo.ZoError) as e:                      # no activation codes: nothing to contract as integers
        zo.zo_linear_fakequant_mma(X, to_dev(W, torch), 4, 64, 16, 1, 0, 0.0)
    assert e.value.status == 5
