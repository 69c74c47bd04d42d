"""Pins for the oracle's reading of a quantized linear whose contraction runs on the integer codes (Config.mma = 1):
the operands are the quantizer's outputs (code - zp) * step un-rounded, so the layer is, exactly,

    y[t, n] = step_x[t] * sum_g step_w[n, g] * sum_{k in g} (qx[t, k] - zx[t]) (qw[n, k] - zw[n, g])

(Background/Quantization: codes and de-quantization; Appendix/Quantization settings: per-token activations, per-group
weights).  The right-hand side is evaluated here with Python integers for the inner sums -- no rounding at all -- and
must agree with the oracle's linear on its own de-quantized operands; the same sum re-centred on activation codes that
fit a signed byte (the form a byte-wide matrix instruction needs) is the same number."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def _factorised(qa, qw, group, offset=None):
    """step_x * sum_g step_w * integer inner sums; with `offset`, activation codes are re-centred to q - offset and the
    rank-one term (offset - zx) * sum_g step_w * sum_k (qw - zw) is added back."""
    cx, cw = qa["codes"].astype(np.int64), qw["codes"].astype(np.int64)
    zx, zw = qa["zp"].astype(np.int64), qw["zp"].astype(np.int64)
    M, K = cx.shape
    N = cw.shape[0]
    G = K // group
    dw = (cw.reshape(N, G, group) - zw[:, :, None])                      # integer weight codes minus zero point
    y = np.zeros((M, N), np.float64)
    if offset is None:
        dx = (cx - zx[:, None]).reshape(M, G, group)
        S = np.einsum("tgk,ngk->tng", dx, dw)                           # exact int64
        y = (S.astype(np.float64) * qw["step"].astype(np.float64)[None, :, :]).sum(-1)
    else:
        dx = (cx - offset).reshape(M, G, group)
        assert dx.min() >= -128 and dx.max() <= 127
        S = np.einsum("tgk,ngk->tng", dx, dw)
        A = (S.astype(np.float64) * qw["step"].astype(np.float64)[None, :, :]).sum(-1)
        R = (dw.sum(-1).astype(np.float64) * qw["step"].astype(np.float64)).sum(-1)          # [N]
        y = A + (offset - zx).astype(np.float64)[:, None] * R[None, :]
    return y * qa["step"].astype(np.float64)[:, None]


@pytest.mark.parametrize("a_bits,w_bits,group", [(8, 4, 64), (4, 4, 32), (8, 2, 64), (8, 8, 128)])
def test_integer_route_is_the_unrounded_operand_product(a_bits, w_bits, group):
    M, N, K = 9, 24, 256
    X = synth.activations((M, K), 31)
    X[3] = np.abs(X[3]) + 0.25                        # an all-positive row: zero point below zero
    W = synth.weights((N, K), 32)
    qa = orc.fakequant_act(X, a_bits)
    qw = orc.fakequant_weight(W, w_bits, group, seed=5, tensor_id=2, eps_signed=np.float32(1e-3))
    y = orc.linear(qa["xhat"], qw["what"])            # operands as the quantizers return them (fp32)
    yi = _factorised(qa, qw, group)
    mag = np.abs(qa["xhat"].astype(np.float64)) @ np.abs(qw["what"].astype(np.float64)).T
    assert np.all(np.abs(y - yi) <= 3e-7 * mag)       # (q - zp) * step is rounded once to fp32 per operand
    yo = _factorised(qa, qw, group, offset=1 << (a_bits - 1))
    assert np.all(np.abs(yo - yi) <= 1e-12 * mag + 1e-12)
    # and it is NOT what bf16-rounded operands give
    yb = orc.linear(orc.bf16_round(qa["xhat"]), orc.bf16_round(qw["what"]))
    assert np.abs(yb - yi).max() > 1e-4 * np.abs(yi).max()


def test_model_forward_mma_switch():
    """mma = 1 changes the operands of the quantized linears in bf16 storage and nothing else: identical to mma = 0 in
    fp32 storage, identical without activation codes, and within the size of the operand rounding otherwise."""
    base = dict(n_layers=2, d_model=64, n_heads=2, d_ffn=128, vocab=128, max_seq=12, w_bits=4, w_group=32)
    ids = synth.token_ids(2, 12, 128, 41)
    for arch in (orc.ARCH_LLAMA, orc.ARCH_OPT):
        shapes = orc.param_shapes(orc.Config(arch, a_bits=8, **base))
        params = synth.model_params(shapes, 40)
        f = lambda **kw: orc.forward(orc.Config(arch, **base, **kw), params, ids=ids, seed=3, eps_signed=np.float32(1e-3))
        assert f(a_bits=8, act_dtype=0, mma=1) == f(a_bits=8, act_dtype=0, mma=0)
        assert f(a_bits=16, act_dtype=1, mma=1) == f(a_bits=16, act_dtype=1, mma=0)
        l1, l0, l32 = f(a_bits=8, act_dtype=1, mma=1), f(a_bits=8, act_dtype=1, mma=0), f(a_bits=8, act_dtype=0, mma=0)
        assert l1 != l0 and abs(l1 - l0) < 2e-3 * abs(l0)
        assert abs(l1 - l32) < 2e-3 * abs(l32)


def test_linear_arch_mma_is_exactly_the_factorised_sum():
    cfg = orc.Config(orc.ARCH_LINEAR, d_model=128, d_ffn=48, w_bits=4, w_group=64, a_bits=8, act_dtype=1, mma=1)
    W = synth.weights((48, 128), 51)
    x = orc.bf16_round(synth.activations((8, 128), 52))
    tgt = synth.activations((8, 48), 53)
    trace = {}
    orc.forward(cfg, [W], x=x, target=tgt, seed=9, eps_signed=np.float32(-1e-3), trace=trace)
    qa = orc.fakequant_act(x, 8)
    qw = orc.fakequant_weight(W, 4, 64, seed=9, tensor_id=0, eps_signed=np.float32(-1e-3))
    want = orc.bf16_round(_factorised(qa, qw, 64).astype(np.float32))     # the stored output is still bf16
    got = trace["y"]
    assert np.mean(got == want) > 0.995 and np.abs(got - want).max() <= 2.0 ** -7 * np.abs(want).max()
