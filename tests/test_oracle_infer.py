"""Pins for the oracle's generator (prompt pass + cached decoding, the inference side of the efficiency section's
on-device table).  Nothing here is compared with itself: the cached path is checked against the training-time forward
(a different code path: batched attention over whole sequences), against recomputing the longer prompt from scratch,
and against causality."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth


def _model(arch, act_dtype, packed, a_bits=8, seed=70):
    base = dict(n_layers=2, d_model=64, n_heads=2, d_ffn=128, vocab=96, max_seq=24, w_bits=4, w_group=32, a_bits=a_bits)
    cfg = orc.Config(arch, act_dtype=act_dtype, lightweight=1 if packed else 0, **base)
    shapes = orc.param_shapes(cfg)
    params = synth.model_params(shapes, seed)
    params = [p * (3.0 if p.ndim == 2 else 1.0) for p in params]
    trainable = None
    if packed:                                     # the trained model as deployed: every quantized linear as 4-bit codes
        trainable = [False] * len(shapes)
        params = [orc.pack_int4(p, 32) if q else p for p, (_, _, q) in zip(params, shapes)]
    return cfg, params, trainable


@pytest.mark.parametrize("arch", [orc.ARCH_LLAMA, orc.ARCH_OPT])
@pytest.mark.parametrize("packed", [False, True])
def test_prompt_pass_equals_the_forward_at_the_last_position(arch, packed):
    cfg, params, trainable = _model(arch, 0, packed)
    ids = synth.token_ids(1, 17, 96, 71)
    trace = {}
    orc.forward(cfg, params, ids=ids, seed=0, eps_signed=0.0, trainable=trainable, trace=trace)
    kv = orc.new_kv(cfg)
    logits = orc.infer_prefill(cfg, params, ids[0], kv, trainable)
    ref = trace["logits"][-1]
    assert np.abs(logits - ref).max() <= 1e-5 * np.abs(ref).max()
    assert kv[0][0].shape == (17, 64) and kv[1][1].shape == (17, 64)
    # the cache holds what the forward stored: keys after the rotary embedding (Llama-shaped), values as projected
    qkv = trace["l1.qkv"]
    assert np.abs(kv[1][0] - qkv[:, 64:128]).max() <= 1e-5 * np.abs(qkv).max()
    assert np.abs(kv[1][1] - qkv[:, 128:]).max() <= 1e-5 * np.abs(qkv).max()


@pytest.mark.parametrize("arch", [orc.ARCH_LLAMA, orc.ARCH_OPT])
@pytest.mark.parametrize("act_dtype", [0, 1])
def test_cached_step_equals_the_uncached_prompt_pass(arch, act_dtype):
    cfg, params, trainable = _model(arch, act_dtype, True, a_bits=4)
    ids = synth.token_ids(1, 14, 96, 72)[0]
    kv = orc.new_kv(cfg)
    orc.infer_prefill(cfg, params, ids[:10], kv, trainable)
    for n in range(10, 14):
        step = orc.infer_decode(cfg, params, ids[n], kv, trainable)
        kv2 = orc.new_kv(cfg)
        full = orc.infer_prefill(cfg, params, ids[:n + 1], kv2, trainable)
        tol = 1e-9 if act_dtype == 0 else 1e-9        # same arithmetic row by row: nothing but fp64 summation order differs
        assert np.abs(step - full).max() <= tol * np.abs(full).max() + 1e-12
        for l in range(cfg.n_layers):
            assert np.array_equal(kv[l][0], kv2[l][0]) and np.array_equal(kv[l][1], kv2[l][1])


def test_cache_is_causal_and_greedy_follows_the_logits():
    cfg, params, trainable = _model(orc.ARCH_LLAMA, 1, True)
    ids = synth.token_ids(1, 12, 96, 73)[0]
    kv_a, kv_b = orc.new_kv(cfg), orc.new_kv(cfg)
    orc.infer_prefill(cfg, params, ids[:8], kv_a, trainable)
    orc.infer_prefill(cfg, params, ids, kv_b, trainable)
    for l in range(cfg.n_layers):                                  # later tokens do not change earlier cache rows
        assert np.array_equal(kv_a[l][0], kv_b[l][0][:8]) and np.array_equal(kv_a[l][1], kv_b[l][1][:8])
    toks, lgs = orc.greedy_generate(cfg, params, ids[:8], 5, trainable)
    assert toks.shape == (5,) and lgs.shape == (5, 96)
    assert np.array_equal(toks, lgs.argmax(-1))
    # generating 5 tokens = a prompt pass over prompt + the first 4 of them
    kv_c = orc.new_kv(cfg)
    again = orc.infer_prefill(cfg, params, np.concatenate([ids[:8], toks[:4]]), kv_c, trainable)
    assert np.abs(again - lgs[4]).max() <= 1e-9 * np.abs(again).max()
