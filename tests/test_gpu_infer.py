"""GPU parity of the generator on the quantized model (zo_prefill / zo_decode / zo_generate_greedy) against the oracle's:
logits of the prompt pass and of cached steps, the cache contents, greedy tokens where the oracle's own top-2 margin
exceeds the logit tolerance, and a cached step against recomputing the longer prompt on the GPU itself."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


def _model(zo, torch, arch, act_dtype, packed, S_max, d_model=128, n_heads=4, a_bits=8, group=64, n_layers=2, d_ffn=256, vocab=512, seed=1400,
           wscale=3.0):
    base = dict(n_layers=n_layers, d_model=d_model, n_heads=n_heads, d_ffn=d_ffn, vocab=vocab, max_seq=S_max, w_bits=4, w_group=group, a_bits=a_bits)
    ocfg = orc.Config(arch, act_dtype=act_dtype, lightweight=1 if packed else 0, **base)
    cfg = zo.make_config(arch, act_dtype=act_dtype, lightweight=1 if packed else 0, **base)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, seed)
    params = [p * (wscale if p.ndim == 2 else 1.0) for p in params]
    trainable = None
    o_params, g_params = list(params), [to_dev(p, torch) for p in params]
    if packed:
        trainable = [False] * len(shapes)
        for i, (w, (_, _, q)) in enumerate(zip(params, shapes)):
            if q:
                o_params[i] = orc.pack_int4(w, group)
                g_params[i] = zo.zo_pack_weight_int4(g_params[i], group)
    ctx = zo.Context(cfg, g_params, 1, S_max, trainable=trainable)
    return ocfg, o_params, trainable, ctx


def _check_logits(got, ref, act_dtype, what):
    """fp32 storage: every logit to 2e-4 of the largest.  bf16 storage with 8-bit activation codes: two valid evaluation
    orders (or operand roundings: the one-token kernel of a decoding step contracts un-rounded de-quantized weights) drift
    apart to about one code step of the activations -- the vector of logits to 2e-2 relative l2, single logits to 5e-2."""
    err = np.abs(got - ref)
    if act_dtype == 0:
        assert err.max() <= 2e-4 * np.abs(ref).max(), (what, err.max(), np.abs(ref).max())
    else:
        assert np.linalg.norm(got - ref) <= 2e-2 * np.linalg.norm(ref), (what, np.linalg.norm(got - ref) / np.linalg.norm(ref))
        assert err.max() <= 5e-2 * np.abs(ref).max(), (what, err.max(), np.abs(ref).max())


@pytest.mark.parametrize("arch", [1, 2])
@pytest.mark.parametrize("act_dtype,packed", [(0, False), (1, False), (1, True)])
def test_prompt_pass_and_cached_steps_vs_oracle(arch, act_dtype, packed):
    torch, zo = gpu()
    S, S_max, n_new = 21, 32, 5
    # (weights three times the usual scale make the fp32 comparison sharp; in bf16 storage that regime amplifies every
    # storage rounding through the 8-bit activation codes, so the usual scale is used there)
    ocfg, o_params, trainable, ctx = _model(zo, torch, arch, act_dtype, packed, S_max, wscale=1.0 if act_dtype else 3.0)
    prompt = synth.token_ids(1, S, 512, 1401)[0]
    extra = synth.token_ids(1, n_new, 512, 1402)[0]
    kv = ctx.new_kv_cache(S_max)
    okv = orc.new_kv(ocfg)
    got = ctx.zo_prefill(to_dev(prompt, torch), kv, S_max).cpu().numpy()
    ref = orc.infer_prefill(ocfg, o_params, prompt, okv, trainable)
    _check_logits(got, ref, act_dtype, "prompt")
    td = torch.bfloat16 if act_dtype else torch.float32
    for i in range(n_new):                                             # teacher-forced: both sides see the same tokens
        tok = to_dev(extra[i:i + 1], torch)
        got = ctx.zo_decode(tok, S + i, kv, S_max).cpu().numpy()
        ref = orc.infer_decode(ocfg, o_params, extra[i], okv, trainable)
        _check_logits(got, ref, act_dtype, i)
    cache = kv.view(td).float().cpu().numpy().reshape(ocfg.n_layers, 2, S_max, ocfg.d_model)
    for l in range(ocfg.n_layers):
        for j in range(2):
            want = okv[l][j]
            err = np.linalg.norm(cache[l, j, :S + n_new] - want) / np.linalg.norm(want)
            assert err <= (2e-2 if act_dtype else 1e-4), (l, j, err)
        assert not cache[l, :, S + n_new:].any()                       # rows past the sequence were never written
    ctx.close()


@pytest.mark.parametrize("arch", [1, 2])
def test_greedy_generation_vs_oracle(arch):
    """fp32 storage so that logits agree to ~1e-5: wherever the oracle's best and second-best logits are further apart
    than that, the generated token must be the oracle's; the run stops comparing at the first step where they are not
    (from there the two sides may legitimately continue with different tokens)."""
    torch, zo = gpu()
    S, S_max, n_new = 12, 32, 12
    ocfg, o_params, trainable, ctx = _model(zo, torch, arch, 0, False, S_max, a_bits=16)
    prompt = synth.token_ids(1, S, 512, 1403)[0]
    kv = ctx.new_kv_cache(S_max)
    toks, _ = ctx.zo_generate_greedy(to_dev(prompt, torch), n_new, kv, S_max)
    toks = toks.cpu().numpy()
    otoks, olgs = orc.greedy_generate(ocfg, o_params, prompt, n_new, trainable)
    checked = 0
    for i in range(n_new):
        top2 = np.sort(olgs[i])[-2:]
        if top2[1] - top2[0] < 1e-3 * np.abs(olgs[i]).max():
            break
        assert toks[i] == otoks[i], (i, toks, otoks)
        checked += 1
    assert checked >= 6
    ctx.close()


def test_cached_step_equals_recomputed_prompt_on_the_gpu():
    """Widths where the packed-codes small-M kernel splits K and the prompt pass takes the batched GEMMs: the logits of a
    cached step against a fresh prompt pass over the longer sequence (bf16 storage: the two take different kernels, so
    they agree to the storage rounding, not bit for bit)."""
    torch, zo = gpu()
    S, S_max = 40, 64
    ocfg, o_params, trainable, ctx = _model(zo, torch, 1, 1, True, S_max, d_model=512, n_heads=4, d_ffn=1024, a_bits=16, group=128, n_layers=2)
    seq = synth.token_ids(1, S + 1, 512, 1404)[0]
    kv = ctx.new_kv_cache(S_max)
    ctx.zo_prefill(to_dev(seq[:S], torch), kv, S_max)
    step = ctx.zo_decode(to_dev(seq[S:S + 1], torch), S, kv, S_max).cpu().numpy()
    kv2 = ctx.new_kv_cache(S_max)
    full = ctx.zo_prefill(to_dev(seq, torch), kv2, S_max).cpu().numpy()
    okv = orc.new_kv(ocfg)
    ref = orc.infer_prefill(ocfg, o_params, seq, okv, trainable)
    # 16-bit activations: with activation codes two valid evaluation orders drift apart to the size of a code step (~3 % at 8 bits)
    tol = 2e-2 * np.abs(ref).max()
    assert np.abs(step - ref).max() <= tol and np.abs(full - ref).max() <= tol, (np.abs(step - ref).max(), np.abs(full - ref).max(), np.abs(ref).max())
    ctx.close()


def test_generator_rejects_bad_requests():
    torch, zo = gpu()
    ocfg, o_params, trainable, ctx = _model(zo, torch, 1, 1, False, 16)
    kv = ctx.new_kv_cache(16)
    ids = to_dev(synth.token_ids(1, 16, 512, 1405)[0], torch)
    with pytest.raises(zo.ZoError):
        ctx.zo_decode(ids[:1], 16, kv, 16)                 # position beyond the cache
    with pytest.raises(zo.ZoError):
        ctx.zo_prefill(ids, kv, 32)                        # cache longer than max_seq
    with pytest.raises(zo.ZoError):
        ctx.zo_generate_greedy(ids[:10], 8, kv, 16)        # 10 + 8 - 1 > 16
    ctx.close()


@pytest.mark.parametrize("a_bits", [8, 4])
def test_generator_at_7b_widths_one_layer(a_bits):
    """One decoder layer of the benchmark's generator workload (d 4096, 32 heads, SwiGLU 11008, vocabulary 32000, every
    quantized linear as packed 4-bit codes in groups of 128, bf16 storage, 384-token prompt): the kernels that workload
    times -- batched GEMMs and matrix-core attention in the prompt pass; the one-token packed-codes linear with q | k | v
    and gate | up in one launch, cached attention over ~400 rows and the fused lm_head in a decoding step.  The cache rows
    (one norm + quantizer and one linear away from the embedding) are held sharply; logits to 5e-2 (relative l2) with 8-bit
    activations; with the workload's 4-bit activations two valid roundings drift apart to a sizeable fraction of the
    signal after three quantizers (see test_gpu_widths.py), so the logits are only required to correlate strongly."""
    torch, zo = gpu()
    S, S_max, n_new = 384, 448, 2
    ocfg, o_params, trainable, ctx = _model(zo, torch, 1, 1, True, S_max, d_model=4096, n_heads=32, a_bits=a_bits, group=128, n_layers=1,
                                            d_ffn=11008, vocab=32000, wscale=1.0)
    prompt = synth.token_ids(1, S, 32000, 1406)[0]
    extra = synth.token_ids(1, n_new, 32000, 1407)[0]
    kv = ctx.new_kv_cache(S_max)
    okv = orc.new_kv(ocfg)

    def check(got, ref, what):
        rel = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
        c = float(np.dot(got, ref) / (np.linalg.norm(got) * np.linalg.norm(ref)))
        print("A%d logits, %s: relative l2 error %.4f, correlation with the oracle %.4f" % (a_bits, what, rel, c))
        # 8-bit codes: a disagreement of e comes out of a quantizer as about sqrt(e * step / 2) with a step of 1/30 of the
        # row's spread, which levels off near 3 % after the layer's three quantizers behind the attention
        assert rel <= 5e-2 if a_bits == 8 else c > 0.8, (what, rel, c)

    got = ctx.zo_prefill(to_dev(prompt, torch), kv, S_max).cpu().numpy()
    check(got, orc.infer_prefill(ocfg, o_params, prompt, okv, trainable), "prompt")
    for i in range(n_new):
        got = ctx.zo_decode(to_dev(extra[i:i + 1], torch), S + i, kv, S_max).cpu().numpy()
        check(got, orc.infer_decode(ocfg, o_params, extra[i], okv, trainable), "step %d" % i)
    cache = kv.view(torch.bfloat16).float().cpu().numpy().reshape(1, 2, S_max, 4096)
    for j in range(2):
        want = okv[0][j]
        err = np.linalg.norm(cache[0, j, :S + n_new] - want, axis=1) / np.linalg.norm(want, axis=1)
        # a row may carry flipped activation codes (its input sat on a rounding boundary); almost every row agrees to rounding
        assert np.median(err) < 5e-3 and np.quantile(err, 0.9) < (2e-2 if a_bits == 8 else 0.2), (j, np.median(err), err.max())
        assert np.median(err[S:]) < (2e-2 if a_bits == 8 else 0.2), (j, err[S:])
    assert not cache[0, :, S + n_new:].any()
    ctx.close()


@pytest.mark.parametrize("arch,act_dtype", [(2, 0), (1, 0), (2, 1)])
def test_cached_steps_over_several_ranges_of_rows(arch, act_dtype):
    """Enough cached rows for the decoding step's attention to split them into ranges (64-wide heads: 32 row groups of 8
    lanes, ranges of 64 rows), with learned positions (no rotation in the kernel) and with the rotary embedding, fp32 and
    bf16 storage: logits of cached steps and the appended cache rows against the oracle."""
    torch, zo = gpu()
    S, S_max, n_new = 150, 160, 3
    ocfg, o_params, trainable, ctx = _model(zo, torch, arch, act_dtype, False, S_max, d_model=256, n_heads=4, a_bits=16, d_ffn=256,
                                            n_layers=1, wscale=1.0)
    prompt = synth.token_ids(1, S, 512, 1408)[0]
    extra = synth.token_ids(1, n_new, 512, 1409)[0]
    kv = ctx.new_kv_cache(S_max)
    okv = orc.new_kv(ocfg)
    ctx.zo_prefill(to_dev(prompt, torch), kv, S_max)
    orc.infer_prefill(ocfg, o_params, prompt, okv, trainable)
    for i in range(n_new):
        got = ctx.zo_decode(to_dev(extra[i:i + 1], torch), S + i, kv, S_max).cpu().numpy()
        ref = orc.infer_decode(ocfg, o_params, extra[i], okv, trainable)
        _check_logits(got, ref, act_dtype, i)
    td = torch.bfloat16 if act_dtype else torch.float32
    cache = kv.view(td).float().cpu().numpy().reshape(1, 2, S_max, 256)
    for j in range(2):
        want = okv[0][j]
        err = np.linalg.norm(cache[0, j, S:S + n_new] - want[S:]) / np.linalg.norm(want[S:])
        assert err <= (2e-2 if act_dtype else 1e-4), (j, err)
    ctx.close()
