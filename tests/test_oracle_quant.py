"""Pins for the oracle's quantizer (CPU only): invariants of the uniform quantizer of the
Background section, special cases with closed-form answers, and the paper's literal formula
evaluated in fp64 (agreement except on flagged rounding ties)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def _literal_fp64(x, bits):
    """clamp(round(X/step) + zp, 0, Q_P) with step=(max-min)/Q_P, zp=-round(min/step), in fp64."""
    x = x.astype(np.float64)
    qp = 2 ** bits - 1
    step = (x.max() - x.min()) / qp
    zp = -np.rint(x.min() / step)
    ratio = x / step
    q = np.clip(np.rint(ratio) + zp, 0, qp)
    frac = np.abs(ratio - np.floor(ratio) - 0.5)
    tie = frac < 1e-6 * np.abs(ratio) + 2.0 ** -20
    return step, zp, q, tie


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("n", [2, 64, 128, 4096])
def test_codes_in_range_and_error_bound(bits, n):
    for seed in range(5):
        x = synth.weights((n,), seed, bits) * (1.0 + seed)
        x[0] += 0.01 * seed                                   # asymmetric range
        step, zp, codes, xhat = orc.quant_group(x, bits)
        qp = 2 ** bits - 1
        assert codes.min() >= 0 and codes.max() <= qp
        assert np.float32(step) == np.float32((x.max() - x.min()) / np.float32(qp))
        assert np.abs(xhat.astype(np.float64) - x).max() <= 0.5 * step * (1 + 1e-5) + 1e-12
        assert codes[np.argmin(x)] in (0, 1) and codes[np.argmax(x)] in (qp - 1, qp)
        assert np.array_equal(xhat, ((codes - zp).astype(np.float32) * np.float32(step)))


@settings(max_examples=200, deadline=None)
@given(st.integers(1, 8), st.integers(2, 200), st.integers(0, 2 ** 31), st.floats(1e-3, 1e3), st.floats(-50, 50))
def test_quantizer_properties_random(bits, n, seed, scale, shift):
    x = (synth.activations((n,), seed) * np.float32(scale) + np.float32(shift * scale)).astype(np.float32)
    step, zp, codes, xhat = orc.quant_group(x, bits)
    qp = 2 ** bits - 1
    assert 0 <= codes.min() and codes.max() <= qp
    if step > 1e-5:
        # values far from 0 lose fp32 resolution in x*inv; bound grows by their rounding error
        slack = 0.5 * step * 1e-4 + np.abs(x).max() * 2.0 ** -22
        assert np.abs(xhat.astype(np.float64) - x).max() <= 0.5 * step + slack


def test_matches_literal_formula_except_flagged_ties():
    mismatches = flagged = total = 0
    for bits in (2, 4, 8):
        for seed in range(40):
            x = synth.weights((64,), seed, 100 + bits)
            step, zp, codes, _ = orc.quant_group(x, bits)
            s64, zp64, q64, tie = _literal_fp64(x, bits)
            assert abs(step - s64) <= 1e-6 * s64
            # where the zero points differ by a tie on min/step every code shifts with them: skip
            if zp != int(zp64):
                continue
            bad = codes != q64.astype(np.int64)
            total += x.size
            mismatches += int(np.sum(bad & ~tie))
            flagged += int(np.sum(bad & tie))
    assert mismatches == 0
    assert flagged <= max(1, total // 1000)


def test_integer_grid_is_reproduced_exactly():
    for bits in (2, 4, 8):
        qp = 2 ** bits - 1
        x = np.arange(qp + 1, dtype=np.float32)
        np.random.default_rng(0).shuffle(x)
        step, zp, codes, xhat = orc.quant_group(x, bits)
        assert step == 1.0 and zp == 0
        assert np.array_equal(codes, x.astype(np.int32)) and np.array_equal(xhat, x)
        # shifted grid: zero-point moves, values still exact
        step, zp, codes, xhat = orc.quant_group(x - 3.0, bits)
        assert step == 1.0 and zp == 3 and np.array_equal(xhat, x - 3.0)


def test_one_bit_two_valued_group():
    # The grid is anchored at multiples of the step (zp = -round(min/step)), not at min:
    # a two-valued group is reproduced exactly iff min is a multiple of the step.
    x = np.array([0.0, -0.75, 0.0, 0.0, -0.75], np.float32)
    step, zp, codes, xhat = orc.quant_group(x, 1)
    assert step == 0.75 and zp == 1 and set(codes.tolist()) == {0, 1}
    assert np.array_equal(xhat, x)
    x = np.array([0.25, -0.5, 0.25, 0.25, -0.5], np.float32)      # min/step = -2/3 -> zp = 1
    step, zp, codes, xhat = orc.quant_group(x, 1)
    assert step == 0.75 and zp == 1
    assert np.array_equal(xhat, np.array([0.0, -0.75, 0.0, 0.0, -0.75], np.float32))
    assert np.abs(xhat - x).max() <= 0.5 * step


def test_all_positive_group_has_zero_point_outside_code_range():
    x = np.linspace(10.0, 11.5, 16).astype(np.float32)          # step 0.1, min/step = 100
    step, zp, codes, xhat = orc.quant_group(x, 4)
    assert zp == -100 and codes.min() == 0 and codes.max() == 15
    assert np.abs(xhat - x).max() <= 0.5 * step * (1 + 1e-4)


def test_constant_group_uses_step_floor():
    x = np.full(64, 0.0123, np.float32)
    step, zp, codes, xhat = orc.quant_group(x, 4)
    assert step == np.float32(1e-5)
    assert np.all(codes == codes[0]) and np.abs(xhat - x).max() <= 1e-5


def test_near_idempotent():
    x = synth.weights((128,), 3)
    _, _, _, xhat = orc.quant_group(x, 4)
    step2, _, _, xhat2 = orc.quant_group(xhat, 4)
    assert np.abs(xhat2 - xhat).max() <= 1e-3 * step2


@pytest.mark.parametrize("bits", [4, 8])
def test_symmetric_variant(bits):
    x = synth.activations((300,), 5)
    step, zp, codes, xhat = orc.quant_group(x, bits, sym=True)
    qp = 2 ** (bits - 1) - 1
    assert zp == 0 and codes.min() >= -qp - 1 and codes.max() <= qp
    assert np.float32(step) == np.float32(np.abs(x).max() / np.float32(qp))
    assert abs(codes[np.argmax(np.abs(x))]) == qp
    assert np.abs(xhat - x).max() <= 0.5 * step * (1 + 1e-4)


def test_weight_groups_are_contiguous_along_in_features():
    # group g of row n covers W[n, g*G:(g+1)*G]; every group equals the 1-group routine
    W = synth.weights((6, 256), 11)
    out = orc.fakequant_weight(W, 4, 64)
    assert out["step"].shape == (6, 4)
    for n in (0, 5):
        for g in range(4):
            step, zp, codes, xhat = orc.quant_group(W[n, g * 64:(g + 1) * 64], 4)
            assert out["step"][n, g] == step and out["zp"][n, g] == zp
            assert np.array_equal(out["codes"][n, g * 64:(g + 1) * 64], codes)
            assert np.array_equal(out["what"][n, g * 64:(g + 1) * 64], xhat)
    # group 0 (or K) = per-channel
    pc = orc.fakequant_weight(W, 4, 0)
    assert pc["step"].shape == (6, 1)
    assert pc["step"][2, 0] == orc.quant_group(W[2], 4)[0]


def test_weight_quantizer_sees_the_perturbed_weights():
    W = synth.weights((4, 128), 12)
    eps = np.float32(1e-3)
    z = orc.normal(77, 9, W.size).reshape(W.shape)
    plus = orc.fakequant_weight(W, 4, 64, seed=77, tensor_id=9, eps_signed=eps)
    minus = orc.fakequant_weight(W, 4, 64, seed=77, tensor_id=9, eps_signed=-eps)
    wp = (W.astype(np.float64) + 1e-3 * z).astype(np.float32)
    wm = (W.astype(np.float64) - 1e-3 * z).astype(np.float32)
    # fused multiply-add vs separately rounded product: at most one ulp apart
    assert np.abs(orc.perturb(W, 77, 9, eps) - wp).max() <= 2 ** -23 * np.abs(W).max() * 2
    assert np.array_equal(plus["what"], orc.fakequant_weight(orc.perturb(W, 77, 9, eps), 4, 64)["what"])
    assert np.array_equal(minus["what"], orc.fakequant_weight(orc.perturb(W, 77, 9, -eps), 4, 64)["what"])
    assert np.abs(orc.perturb(W, 77, 9, -eps) - wm).max() <= 2 ** -23 * np.abs(W).max() * 2
    # bits = 0: perturbed, not quantized
    assert np.array_equal(orc.fakequant_weight(W, 0, 0, 77, 9, eps)["what"], orc.perturb(W, 77, 9, eps))


def test_per_token_activation_rows_are_independent_groups():
    X = synth.activations((5, 96), 13)
    out = orc.fakequant_act(X, 8)
    for m in range(5):
        step, zp, codes, xhat = orc.quant_group(X[m], 8)
        assert out["step"][m] == step and out["zp"][m] == zp
        assert np.array_equal(out["codes"][m], codes) and np.array_equal(out["xhat"][m], xhat)
    assert np.array_equal(orc.fakequant_act(X, 16)["xhat"], X)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -8 + 2 ** -20, -3.1415927, 0.0, 1e-30, 65504.0], np.float32)
    got = orc.bf16_round(x)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == np.float32(1.015625)
    assert got[3] == np.float32(1.0078125)
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, ref)
    big = synth.activations((10000,), 14) * 37.0
    assert np.array_equal(orc.bf16_round(big), torch.from_numpy(big).to(torch.bfloat16).float().numpy())


def test_linear_triple_loop_matches_library_matmul():
    x = synth.activations((7, 40), 15)
    w = synth.weights((9, 40), 16)
    b = synth.weights((9,), 17)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    assert np.allclose(orc.linear(x, w, b), ref, rtol=1e-13, atol=1e-15)
    # a transposed operand or a dropped bias would fail these
    assert not np.allclose(orc.linear(x, w), ref, rtol=1e-6)
