"""Pins of the oracle's frozen, pre-quantized weight format (lightweight variant: Section
"Lightweight ZeroQAT for memory reduction"): binary16 conversion against numpy's, nibble order on a
hand-written example, exact reproduction of on-grid matrices, the error bound of the stored form,
and the model forward with packed tensors against the same forward on fp32 copies."""
import numpy as np

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def test_f16_conversion_matches_numpy():
    rng = synth.rng(301)
    x = (rng.standard_normal(100000) * 10.0 ** rng.integers(-9, 6, 100000)).astype(np.float32)
    edge = np.array([0.0, -0.0, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 2.0 ** -24, 1.5 * 2.0 ** -24,
                     2.5 * 2.0 ** -24, 2.0 ** -14, np.nextafter(np.float32(2.0 ** -14), np.float32(0)), 65504.0, 65519.0, 65520.0,
                     1e6, -1e-5, 1e-5, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, np.inf, -np.inf], np.float32)
    x = np.concatenate([x, edge])
    got = np.array([orc.f32_to_f16_bits(v) for v in x], np.uint16)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)
    hs = np.array([h for h in range(65536) if (h >> 10) & 31 != 31], np.uint16)
    back = np.array([orc.f16_bits_to_f32(h) for h in hs], np.float32)
    assert np.array_equal(back.view(np.uint32), hs.view(np.float16).astype(np.float32).view(np.uint32))


def test_nibble_order_and_exact_grid():
    # one channel, one group of 16: w_k = k/2 -> step 1/2 (exact in binary16), zero point 0, code k
    W = (np.arange(16, dtype=np.float32) * np.float32(0.5)).reshape(1, 16)
    p = orc.pack_int4(W, 16)
    assert p.codes.tolist() == [[0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]]
    assert p.step_f16.tolist() == [[0x3800]] and p.zp.tolist() == [[0]]
    assert np.array_equal(orc.dequant_int4(p), W)


def test_shifted_grid_reproduced_exactly():
    rng = synth.rng(302)
    N, K, g = 6, 64, 32
    codes = rng.integers(0, 16, (N, K))
    codes[:, ::g] = 0
    codes[:, 1::g] = 15                                  # both end codes present in every group
    zp = rng.integers(0, 16, (N, K // g))
    step = np.float32(2.0) ** rng.integers(-9, -3, (N, K // g)).astype(np.float32)
    W = ((codes - np.repeat(zp, g, 1)) * np.repeat(step, g, 1)).astype(np.float32)
    p = orc.pack_int4(W, g)
    assert np.array_equal(p.zp, zp.astype(np.int16))
    assert np.array_equal(p.step_f16.view(np.float16).astype(np.float32), step)
    lo, hi = p.codes & 15, p.codes >> 4
    assert np.array_equal(lo, codes[:, 0::2]) and np.array_equal(hi, codes[:, 1::2])
    assert np.array_equal(orc.dequant_int4(p), W)
    # an on-grid matrix is a fixed point of the fake-quantizer too: both routes give the same operand
    assert np.array_equal(orc.fakequant_weight(W, 4, g)["what"], W)


def test_stored_form_error_bound_and_relation_to_fake_quantizer():
    W = synth.weights((32, 256), 303)
    g = 128
    p = orc.pack_int4(W, g)
    fq = orc.fakequant_weight(W, 4, g)
    # same codes and zero points as the fake-quantizer at eps = 0
    codes = np.empty((32, 256), np.int32)
    codes[:, 0::2], codes[:, 1::2] = p.codes & 15, p.codes >> 4
    assert np.array_equal(codes, fq["codes"]) and np.array_equal(p.zp.astype(np.int32), fq["zp"])
    step16 = p.step_f16.view(np.float16).astype(np.float32)
    assert np.all(np.abs(step16 - fq["step"]) <= fq["step"] * 2.0 ** -11)          # binary16 rounding of the step
    what = orc.dequant_int4(p)
    want = ((codes - np.repeat(fq["zp"], g, 1)).astype(np.float32) * np.repeat(step16, g, 1)).astype(np.float32)
    assert np.array_equal(what, want)
    # distance to the original weight: half a step plus the step's own rounding times the code distance
    bound = np.repeat(fq["step"], g, 1) * (0.5 + 1e-5) + np.abs(codes - np.repeat(fq["zp"], g, 1)) * np.repeat(np.abs(step16 - fq["step"]), g, 1)
    assert np.all(np.abs(what - W) <= bound + 1e-9)
    # bf16 operand rounding
    assert np.array_equal(orc.dequant_int4(p, round_bf16=True), orc.bf16_round(what))


def _on_grid(shape, g, seed):
    rng = synth.rng(seed)
    N, K = shape
    codes = rng.integers(0, 16, (N, K))
    codes[:, ::g] = 0
    codes[:, 1::g] = 15
    zp = rng.integers(5, 11, (N, K // g))
    step = np.float32(2.0) ** rng.integers(-8, -6, (N, K // g)).astype(np.float32)
    return ((codes - np.repeat(zp, g, 1)) * np.repeat(step, g, 1)).astype(np.float32)


def test_model_forward_with_packed_tensors_equals_fp32_frozen_route():
    cfg = orc.Config(orc.ARCH_LLAMA, n_layers=2, d_model=64, n_heads=2, d_ffn=128, vocab=97, max_seq=16,
                     w_bits=4, w_group=32, a_bits=8, act_dtype=0, lightweight=1)
    shapes = orc.param_shapes(cfg)
    params, trainable = [], []
    for i, (name, shape, quantized) in enumerate(shapes):
        tr = name.endswith(".wq") or name.endswith(".wv")
        trainable.append(tr)
        if quantized and not tr:
            params.append(_on_grid(shape, 32, 400 + i))          # frozen linears: exactly on a 4-bit grid
        elif len(shape) == 1:
            params.append(np.ones(shape, np.float32))
        else:
            params.append(synth.weights(shape, 400 + i))
    ids = synth.token_ids(2, 16, 97, 7)
    packed = [orc.pack_int4(w, 32) if (q and not t) else w for w, t, (_, _, q) in zip(params, trainable, shapes)]
    for eps in (0.0, 1e-3, -1e-3):
        a = orc.forward(cfg, params, ids=ids, seed=3, eps_signed=eps, trainable=trainable)
        b = orc.forward(cfg, packed, ids=ids, seed=3, eps_signed=eps, trainable=trainable)
        assert a == b
    # a step leaves packed tensors alone and moves the trainable ones
    before = [w.copy() if isinstance(w, np.ndarray) else w for w in packed]
    lp, lm, g = orc.zo_step(cfg, packed, 3, 1e-3, 1e-2, ids=ids, trainable=trainable)
    assert g != 0
    for w0, w1, t in zip(before, packed, trainable):
        if isinstance(w1, orc.PackedInt4):
            assert w1 is w0
        elif t:
            assert not np.array_equal(w0, w1)
        else:
            assert np.array_equal(w0, w1)
