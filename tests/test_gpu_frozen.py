"""GPU parity of the frozen, pre-quantized weights of the lightweight variant (Section "Lightweight
ZeroQAT for memory reduction"): packing is bit-exact against the oracle (integer codes, binary16
steps, int16 zero points), the de-quantized operand is bit-exact, the frozen linear agrees to the
layer tolerance (1e-4 fp32 storage, 1e-2 bf16), and a lightweight ZO step with packed tensors
matches the oracle's step: packed tensors untouched, Q and V updated bit-exactly."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev, rel_l2

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,K,group", [(24, 256, 128), (7, 192, 64), (130, 1024, 128), (5, 64, 8), (3, 1024, 512)])
def test_pack_is_bit_exact(N, K, group):
    torch, zo = gpu()
    W = synth.weights((N, K), 501)
    if N > 4:
        W[1] = np.abs(W[1]) + 0.5            # a channel whose groups do not straddle zero: zero point outside 0..15
        W[2] = 0.25                          # constant groups: step floored
    p = zo.zo_pack_weight_int4(to_dev(W, torch), group)
    ref = orc.pack_int4(W, group)
    assert np.array_equal(p.codes.cpu().numpy(), ref.codes)
    assert np.array_equal(p.step_f16.view(torch.int16).cpu().numpy().view(np.uint16), ref.step_f16)
    assert np.array_equal(p.zp.cpu().numpy(), ref.zp)


@pytest.mark.parametrize("dtype", ["float32", "bfloat16"])
@pytest.mark.parametrize("a_bits", [16, 8, 4])
def test_frozen_linear(dtype, a_bits):
    torch, zo = gpu()
    M, N, K, group = 150, 200, 384, 128
    tdt = getattr(torch, dtype)
    bf = dtype == "bfloat16"
    W = synth.weights((N, K), 502)
    X = synth.activations((M, K), 503)
    if bf:
        X = orc.bf16_round(X)
    ref_p = orc.pack_int4(W, group)
    packed = zo.PackedInt4(to_dev(ref_p.codes, torch), to_dev(ref_p.step_f16.view(np.int16), torch).view(torch.float16),
                           to_dev(ref_p.zp, torch), N, K, group)
    bias = synth.weights((N,), 504)
    Y, what = zo.zo_linear_frozen_int4(to_dev(X, torch, tdt), packed, to_dev(bias, torch), a_bits)
    what_ref = orc.dequant_int4(ref_p, round_bf16=bf)
    assert np.array_equal(what.float().cpu().numpy().view(np.uint32), what_ref.view(np.uint32))
    xq = orc.fakequant_act(X, a_bits, 0, round_bf16=bf, want_codes=False)["xhat"] if a_bits < 16 else X
    ref = orc.linear(xq, what_ref, bias)
    assert rel_l2(Y.float().cpu().numpy(), ref) < (1e-2 if bf else 1e-4)


def test_attach_rejects_bad_requests():
    torch, zo = gpu()
    base = dict(n_layers=1, d_model=128, n_heads=4, d_ffn=256, vocab=64, max_seq=8, w_bits=4, w_group=64, a_bits=8)
    cfg = zo.make_config(1, act_dtype=0, lightweight=1, **base)
    ocfg = orc.Config(1, act_dtype=0, lightweight=1, **base)
    shapes = orc.param_shapes(ocfg)
    params = [to_dev(p, torch) for p in synth.model_params(shapes, 505)]
    names = [n for n, _, _ in shapes]
    trainable = [n.endswith(".wq") or n.endswith(".wv") for n in names]
    ctx = zo.Context(cfg, params, 1, 8, trainable=trainable)
    wk, wq, norm = names.index("l0.wk"), names.index("l0.wq"), names.index("l0.attn_norm")
    good = zo.zo_pack_weight_int4(params[wk], 64)
    ctx.zo_attach_frozen_int4(wk, good)
    for index, p in ((wq, good), (norm, good), (len(params), good), (-1, good)):
        with pytest.raises(zo.ZoError):
            ctx.zo_attach_frozen_int4(index, p)
    bad = zo.PackedInt4(good.codes, good.step_f16, good.zp, good.N, good.K, 48)
    with pytest.raises(zo.ZoError):
        ctx.zo_attach_frozen_int4(wk, bad)
    ctx.close()
    # a tensor with no storage at all is refused when a forward is asked for
    missing = list(params)
    missing[wk] = zo.PackedInt4(good.codes, good.step_f16, good.zp, good.N, good.K, 64)
    ctx = zo.Context(cfg, missing, 1, 8, trainable=trainable)
    ctx.close()
    with pytest.raises(zo.ZoError):
        zo.Context(zo.make_config(1, act_dtype=0, lightweight=0, **base), missing, 1, 8)


@pytest.mark.parametrize("arch", [1, 2])
@pytest.mark.parametrize("act_dtype,a_bits", [(0, 16), (0, 8), (1, 4)])
def test_lightweight_step_with_packed_tensors(arch, act_dtype, a_bits):
    torch, zo = gpu()
    B, S = 2, 24
    base = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=256, vocab=512, max_seq=S, w_bits=4, w_group=64, a_bits=a_bits)
    ocfg = orc.Config(arch, act_dtype=act_dtype, lightweight=1, **base)
    cfg = zo.make_config(arch, act_dtype=act_dtype, lightweight=1, **base)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 506)
    params = [p * (3.0 if p.ndim == 2 else 1.0) for p in params]
    trainable = [n.endswith(".wq") or n.endswith(".wv") for n, _, _ in shapes]
    ids = synth.token_ids(B, S, 512, 507)
    o_params, g_params = [], []
    for w, t, (_, _, q) in zip(params, trainable, shapes):
        if q and not t:
            o_params.append(orc.pack_int4(w, 64))
            g_params.append(zo.zo_pack_weight_int4(to_dev(w, torch), 64))
        else:
            o_params.append(w.copy())
            g_params.append(to_dev(w, torch))
    ctx = zo.Context(cfg, g_params, B, S, trainable=trainable)
    idd = to_dev(ids, torch)
    loss0 = ctx.zo_forward_quant(idd, None, B, S, seed=4, eps_signed=0.0).item()
    ref0 = orc.forward(ocfg, o_params, ids=ids, seed=4, eps_signed=0.0, trainable=trainable)
    assert abs(loss0 - ref0) <= (3e-3 if act_dtype else 1e-3) * abs(ref0)
    out = ctx.zo_step(idd, None, B, S, seed=4, eps=1e-3, lr=1e-2).cpu().numpy()
    before = [w.copy() if isinstance(w, np.ndarray) else w for w in o_params]
    lp, lm, g = orc.zo_step(ocfg, o_params, 4, 1e-3, 1e-2, ids=ids, trainable=trainable)
    tol = 3e-3 if act_dtype else 1e-3
    assert abs(out[0] - lp) <= tol * abs(lp) and abs(out[1] - lm) <= tol * abs(lm)
    if act_dtype == 0 and a_bits == 16:
        # with quantized activations a code at a rounding boundary may differ between the fp32 path and the
        # fp64 oracle, which moves a loss by ~1e-5 and g = (L+ - L-) / 2 eps by 1e-2; g is held strictly
        # only where no activation code is decided
        assert abs(out[2] - g) <= 1e-3 * abs(g) + 5e-3
    assert out[2] == orc.projected_grad(np.float32(out[0]), np.float32(out[1]), np.float32(1e-3))
    for i, w0 in enumerate(before):
        if isinstance(w0, orc.PackedInt4):
            assert np.array_equal(g_params[i].codes.cpu().numpy(), w0.codes)      # frozen storage untouched
        elif trainable[i]:
            assert np.array_equal(g_params[i].cpu().numpy(), orc.update(w0.copy(), 4, i, np.float32(out[3])))
        else:
            assert np.array_equal(g_params[i].cpu().numpy(), w0)
    ctx.close()


def _packed(zo, torch, ref_p, N, K, group):
    return zo.PackedInt4(to_dev(ref_p.codes, torch), to_dev(ref_p.step_f16.view(np.int16), torch).view(torch.float16),
                         to_dev(ref_p.zp, torch), N, K, group)


@pytest.mark.parametrize("K,group", [(128, 32), (128, 64), (128, 128), (512, 256), (512, 512)])
def test_frozen_fused_operand_bit_exact(K, group):
    """Small-M kernel that expands the packed codes in registers: with one-hot activations it returns its operand."""
    torch, zo = gpu()
    N = 48
    W = synth.weights((N, K), 511)
    W[1] = np.abs(W[1]) + 0.5
    ref_p = orc.pack_int4(W, group)
    what = orc.dequant_int4(ref_p, round_bf16=True)
    packed = _packed(zo, torch, ref_p, N, K, group)
    for k0 in range(0, K, 128):
        X = torch.zeros((128, K), dtype=torch.bfloat16, device="cuda")
        X[:, k0:k0 + 128] = torch.eye(128, dtype=torch.bfloat16, device="cuda")
        for relayout in (False, True):
            Yp, Ym = zo.zo_linear_frozen_int4_fused(X, X, packed, relayout=relayout)
            assert np.array_equal(Yp.float().cpu().numpy().T, what[:, k0:k0 + 128])
            assert torch.equal(Yp, Ym)


@pytest.mark.parametrize("M,N,K,group", [(1, 16, 128, 128), (8, 256, 256, 64), (33, 80, 1024, 128), (100, 272, 5120, 128),
                                         (128, 64, 13824, 128), (60, 160, 992, 32), (128, 512, 1024, 256)])
@pytest.mark.parametrize("out_f32,relayout", [(False, False), (True, True)])
def test_frozen_fused_linear_vs_oracle(M, N, K, group, out_f32, relayout):
    torch, zo = gpu()
    Xp = orc.bf16_round(synth.activations((M, K), 512))
    Xm = orc.bf16_round(synth.activations((M, K), 513))
    W = synth.weights((N, K), 514)
    bias = synth.weights((N,), 515)
    ref_p = orc.pack_int4(W, group)
    what = orc.dequant_int4(ref_p, round_bf16=True)
    Yp, Ym = zo.zo_linear_frozen_int4_fused(to_dev(Xp, torch, torch.bfloat16), to_dev(Xm, torch, torch.bfloat16),
                                            _packed(zo, torch, ref_p, N, K, group), to_dev(bias, torch), out_f32=out_f32,
                                            relayout=relayout)
    for Y, X in ((Yp, Xp), (Ym, Xm)):
        ref = orc.linear(X, what, bias)
        got = Y.float().cpu().numpy()
        mag = np.abs(X.astype(np.float64)) @ np.abs(what.astype(np.float64)).T + np.abs(bias)
        assert np.all(np.abs(got - ref) <= 2.0 ** -20 * mag + (2.0 ** -8 * np.abs(ref) if not out_f32 else 0.0) + 1e-30)
    with pytest.raises(zo.ZoError):
        zo.zo_linear_frozen_int4_fused(torch.zeros((129, K), dtype=torch.bfloat16, device="cuda"), None,
                                       _packed(zo, torch, ref_p, N, K, group))


@pytest.mark.parametrize("arch", [1, 2])
def test_lightweight_step_small_batch_routes(arch):
    """48 tokens, bf16: the trainable Q / V go through the kernel that builds their tiles from the masters, the packed
    tensors through the one that expands the codes; same losses as the quantize-once route, same update."""
    torch, zo = gpu()
    B, S = 2, 24
    base = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=256, vocab=512, max_seq=S, w_bits=4, w_group=64, a_bits=8)
    ocfg = orc.Config(arch, act_dtype=1, lightweight=1, **base)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 516)
    trainable = [n.endswith(".wq") or n.endswith(".wv") for n, _, _ in shapes]
    ids = to_dev(synth.token_ids(B, S, 512, 517), torch)
    outs, ws = [], []
    for no_fused in (0, 1):
        cfg = zo.make_config(arch, act_dtype=1, lightweight=1, no_fused=no_fused, **base)
        g_params = [zo.zo_pack_weight_int4(to_dev(w, torch), 64) if (q and not t) else to_dev(w, torch)
                    for w, t, (_, _, q) in zip(params, trainable, shapes)]
        ctx = zo.Context(cfg, g_params, B, S, trainable=trainable)
        ctx.zo_profile_begin()
        outs.append(ctx.zo_step(ids, None, B, S, seed=6, eps=1e-3, lr=1e-2).cpu().numpy().copy())
        prof = ctx.zo_profile_end()
        assert ctx.zo_debug_routes() & ~zo.ROUTE_GEMM_SPLIT_K == (0 if no_fused else zo.ROUTE_FUSED_SMALL_M | zo.ROUTE_FUSED_INT4)
        n_packed = (5 if arch == 1 else 4) * base["n_layers"]          # every linear but Q and V
        n_master = base["n_layers"] + 1                                 # Q and V of a layer share one launch; the lm_head
        assert prof["fused_int4_linear"][1] == (0 if no_fused else n_packed)
        assert prof["fused_linear"][1] == (0 if no_fused else n_master)
        assert prof["gemm"][1] == (4 * base["n_layers"] + 1 if no_fused else 0)
        ws.append([p.cpu().numpy() for p in g_params if not isinstance(p, zo.PackedInt4)])
        ctx.close()
    assert np.allclose(outs[0][:2], outs[1][:2], rtol=3e-4)
    names = [n for (n, _, _), p in zip(shapes, [None] * len(shapes))]
    k = 0
    for i, ((n, _, q), t) in enumerate(zip(shapes, trainable)):
        if q and not t:
            continue
        if t:       # moved exactly by its own coefficient in both runs
            for r in (0, 1):
                assert np.array_equal(ws[r][k], orc.update(params[i].copy(), 6, i, np.float32(outs[r][3])))
        else:
            assert np.array_equal(ws[0][k], params[i])
        k += 1


@pytest.mark.parametrize("S", [24, 8])
def test_lightweight_small_batch_two_packed_tensors_with_k_split(S):
    """Wide enough (d_model 512, groups of 64: 8 slabs along K) that the packed-codes kernel splits K for the gate | up
    pair -- two packed tensors applied to one input, one launch after the other, each with fp32 partial sums in scratch --
    and for the down projection, with both branches of Eq. 2 in flight.  The activations' fragment-ordered copies of the
    two branches and the partial sums must not share memory: L+ and L- against the oracle and against the
    quantize-once route."""
    torch, zo = gpu()
    B = 2
    base = dict(n_layers=2, d_model=512, n_heads=4, d_ffn=1024, vocab=512, max_seq=S, w_bits=4, w_group=64, a_bits=8)
    ocfg = orc.Config(1, act_dtype=1, lightweight=1, **base)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 518)
    trainable = [n.endswith(".wq") or n.endswith(".wv") for n, _, _ in shapes]
    ids = synth.token_ids(B, S, 512, 519)
    o_params = [orc.pack_int4(w, 64) if (q and not t) else w.copy() for w, t, (_, _, q) in zip(params, trainable, shapes)]
    lp = orc.forward(ocfg, o_params, ids=ids, seed=6, eps_signed=np.float32(1e-3), trainable=trainable)
    lm = orc.forward(ocfg, o_params, ids=ids, seed=6, eps_signed=np.float32(-1e-3), trainable=trainable)
    outs = []
    for no_fused in (0, 1):
        cfg = zo.make_config(1, act_dtype=1, lightweight=1, no_fused=no_fused, **base)
        g_params = [zo.zo_pack_weight_int4(to_dev(w, torch), 64) if (q and not t) else to_dev(w, torch)
                    for w, t, (_, _, q) in zip(params, trainable, shapes)]
        ctx = zo.Context(cfg, g_params, B, S, trainable=trainable)
        outs.append(ctx.zo_step(to_dev(ids, torch), None, B, S, seed=6, eps=1e-3, lr=0.0).cpu().numpy().copy())
        if not no_fused:
            assert ctx.zo_debug_routes() & zo.ROUTE_FUSED_INT4
        ctx.close()
    # 14 or 46 loss positions only: a flipped 8-bit activation code (bf16 storage) moves their mean by up to ~1e-3 relative;
    # activations read from memory that another launch overwrote would move it by tens of per cent
    for out in outs:
        assert abs(out[0] - lp) <= 2e-3 * abs(lp) and abs(out[1] - lm) <= 2e-3 * abs(lm), (out, lp, lm)
    assert np.allclose(outs[0][:2], outs[1][:2], rtol=1e-3)


@pytest.mark.parametrize("N,K,group", [(16, 128, 128), (4, 32, 32), (260, 4096, 64), (1024, 11008, 128), (512, 5120, 512), (64, 13824, 128)])
def test_frozen_linear_for_one_token(N, K, group):
    """The matrix-vector kernel of a decoding step against the definition sum_k x (code - zp) step on UN-rounded
    de-quantized weights (fp64), to the fp32 accumulation bound; K spans fewer chunks than lanes, a ragged number of
    chunks, and several sweeps; with bias, ReLU and residual; an all-positive channel (zero point below zero)."""
    torch, zo = gpu()
    x = orc.bf16_round(synth.activations((1, K), 520))
    W = synth.weights((N, K), 521)
    W[1] = np.abs(W[1]) + 0.5
    bias = synth.weights((N,), 522)
    res = orc.bf16_round(synth.activations((1, N), 523))[0]
    ref_p = orc.pack_int4(W, group)
    what = orc.dequant_int4(ref_p, round_bf16=False)
    packed = _packed(zo, torch, ref_p, N, K, group)
    xd = to_dev(x[0], torch, torch.bfloat16)
    mag = np.abs(x.astype(np.float64)) @ np.abs(what.astype(np.float64)).T
    plain = orc.linear(x, what)[0]
    got = zo.zo_linear_frozen_int4_token(xd, packed, out_f32=True).cpu().numpy()
    # the kernel sums x (128 + code) and removes (128 + zp) sum x afterwards: the bound carries that magnitude
    step = ref_p.step_f16.view(np.float16).astype(np.float64)
    big = np.abs(x.astype(np.float64)).sum() * (128.0 + np.abs(ref_p.zp).max() + 15.0) * step.max()
    assert np.all(np.abs(got - plain) <= 2.0 ** -20 * (mag[0] + big)), np.abs(got - plain).max()
    full = np.maximum(plain + bias, 0.0) + res
    got = zo.zo_linear_frozen_int4_token(xd, packed, bias=to_dev(bias, torch), residual=to_dev(res, torch, torch.bfloat16), relu=True).float().cpu().numpy()
    assert np.all(np.abs(got - full) <= 2.0 ** -8 * np.abs(full) + 2.0 ** -20 * (mag[0] + big) + 1e-6)
