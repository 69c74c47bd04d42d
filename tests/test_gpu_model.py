"""GPU parity: whole quantized forward (loss), and the full ZO step (L+, L-, g, updated weights)
against the oracle on seeded inputs.  Tolerances: losses 1e-3 relative; g 1e-3 relative in fp32
storage mode (in bf16 mode g is a difference of two losses that agree to ~1e-3 and inherits the
bf16 rounding noise of every stored activation; the test bounds it against that noise)."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev, rel_l2

pytestmark = pytest.mark.gpu

ARCHS = {"llama": 1, "opt": 2}


def _setup(zo, torch, arch, act_dtype, B, S, wscale=3.0, **kw):
    base = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=256, vocab=509 + 3, max_seq=S, w_bits=4, w_group=64, a_bits=8)
    base.update(kw)
    ocfg = orc.Config(ARCHS[arch], act_dtype=act_dtype, **base)
    cfg = zo.make_config(ARCHS[arch], act_dtype=act_dtype, **base)
    params = synth.model_params(orc.param_shapes(ocfg), 61)
    params = [p * (wscale if p.ndim == 2 else 1.0) for p in params]
    ids = synth.token_ids(B, S, base["vocab"], 62)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    return ocfg, params, ids, gp, ctx


TIE_MARGIN = 1e-4      # code units; fp32 round-off of the GPU's activations is ~4e-5 code units at 8 bits


def _clean_rows(tie_log, B, S):
    """Rows whose value cannot have been touched by a rounding tie of an activation code: a code
    is decided from an fp32 activation that differs in its last bits between the two sides, so a
    row within TIE_MARGIN of a rounding boundary (as flagged by the oracle alone) may legitimately
    come out one code apart; causal attention carries the difference to later positions."""
    dirty = np.zeros(B * S, bool)
    for m in tie_log:
        dirty |= m < TIE_MARGIN
    dirty = np.maximum.accumulate(dirty.reshape(B, S), axis=1).reshape(-1)
    return ~dirty


def _row_rel(a, b):
    return np.linalg.norm(a.astype(np.float64) - b, axis=1) / np.maximum(np.linalg.norm(b, axis=1), 1e-30)


@pytest.mark.parametrize("arch", ["llama", "opt"])
@pytest.mark.parametrize("act_dtype", [0, 1])
@pytest.mark.parametrize("a_bits", [16, 8])
def test_forward_loss_and_layer_outputs(arch, act_dtype, a_bits):
    _check_forward(arch, act_dtype, a_bits, 3, 40)


@pytest.mark.parametrize("arch", ["llama", "opt"])
@pytest.mark.parametrize("act_dtype", [0, 1])
@pytest.mark.parametrize("d_model,n_heads", [(1280, 10), (4224, 33)])
def test_forward_wide_rows(arch, act_dtype, d_model, n_heads):
    """Rows longer than 1024 elements: the norm + quantizer kernel gives a row to a whole workgroup (one chunk of 2048
    elements per row, partly filled, and three of four).  The sharp check is q | k | v of the layer, one norm +
    quantizer and one linear away from the embedding: almost every row agrees to rounding, a row may carry a flipped
    activation code (4224 elements per row make a value near a rounding tie likely).  Further down, in bf16 storage
    with head dimension 128, the bf16 probabilities of the matrix-core attention (2e-3 per row) flip codes of the
    quantizers that follow in most rows, so only a loose bound holds there."""
    torch, zo = gpu()
    B, S = 2, 20
    ocfg, params, ids, gp, ctx = _setup(zo, torch, arch, act_dtype, B, S, wscale=1.0, n_layers=1, d_model=d_model,
                                        n_heads=n_heads, d_ffn=1536, vocab=512)
    loss = ctx.zo_forward_quant(to_dev(ids, torch), None, B, S, seed=9, eps_signed=1e-3).item()
    trace = {}
    ref = orc.forward(ocfg, params, ids=ids, seed=9, eps_signed=np.float32(1e-3), trace=trace)
    assert abs(loss - ref) <= 2e-3 * abs(ref), (loss, ref)
    td = torch.bfloat16 if act_dtype else torch.float32
    qkv = ctx.zo_debug_buffer(3).view(td).float().cpu().numpy().reshape(B * S, -1)
    err = _row_rel(qkv, trace["l0.qkv"])
    assert np.median(err) < 5e-6 and np.quantile(err, 0.8) < 1e-3 and err.max() < 0.05, (np.median(err), err.max())
    for which, name in ((4, "l0.attn"), (2, "l0.out"), (0, "final")):
        got = ctx.zo_debug_buffer(which).view(td).float().cpu().numpy().reshape(B * S, -1)
        err = _row_rel(got, trace[name])
        assert np.median(err) < (5e-2 if act_dtype else 5e-3) and err.max() < 0.1, (name, np.median(err), err.max())
    ctx.close()


def _check_forward(arch, act_dtype, a_bits, B, S, eps_list=(1e-3, -1e-3, 0.0), **kw):
    torch, zo = gpu()
    ocfg, params, ids, gp, ctx = _setup(zo, torch, arch, act_dtype, B, S, a_bits=a_bits, **kw)
    idd = to_dev(ids, torch)
    tol = 1e-2 if act_dtype else 1e-4
    for eps in eps_list:
        loss = ctx.zo_forward_quant(idd, None, B, S, seed=9, eps_signed=eps).item()
        trace, ties = {}, []
        ref = orc.forward(ocfg, params, ids=ids, seed=9, eps_signed=np.float32(eps), trace=trace, tie_log=ties)
        assert abs(loss - ref) <= 1e-3 * abs(ref), (loss, ref)
        td = torch.bfloat16 if act_dtype else torch.float32
        x = ctx.zo_debug_buffer(2).view(td).float().cpu().numpy().reshape(B * S, -1)
        h = ctx.zo_debug_buffer(0).view(td).float().cpu().numpy().reshape(B * S, -1)
        lg = ctx.zo_debug_buffer(1).view(torch.float32).cpu().numpy().reshape(B * S, -1)
        clean = _clean_rows(ties, B, S)
        if a_bits == 16:
            assert clean.all()                       # weight codes come from identical fp32 inputs
        for got, name in ((x, "l%d.out" % (ocfg.n_layers - 1)), (h, "final"), (lg, "logits")):
            err = _row_rel(got, trace[name])
            if act_dtype == 0:
                # fp32 storage: every row that no flagged tie can have touched is within 1e-4
                if clean.any():
                    assert err[clean].max() < tol, (name, err[clean].max())
                assert np.median(err) < 1e-5, (name, np.median(err))
            elif a_bits == 16:
                assert err.max() < tol, (name, err.max())
            else:
                # bf16 storage: activation codes are decided from bf16 values, identical on both
                # sides unless a storage rounding upstream fell on the other side of a tie
                assert np.median(err) < 1e-3 and np.quantile(err, 0.75) < tol, (name, np.quantile(err, 0.75))
            assert err.max() < 0.1, (name, err.max())        # one flipped code moves a row by step/|row|
    ctx.close()


@pytest.mark.parametrize("arch", ["llama", "opt"])
def test_forward_with_split_k_gemms(arch):
    """A couple of hundred tokens, narrow d_model, long d_ffn: the down projection (and nothing else) runs with its K split
    into ranges whose fp32 partial sums a second kernel adds; same checks as the other bf16 forwards.  (16-bit activations:
    with activation codes, 200 keys and head dimension 64 the bf16 probabilities of the matrix-core attention flip codes in
    most rows, and only a loose bound would hold.)"""
    a_bits = 16
    torch, zo = gpu()
    B, S = 1, 200
    kw = dict(n_layers=1, d_model=256, n_heads=4, d_ffn=2048, vocab=512)
    _check_forward(arch, 1, a_bits, B, S, eps_list=(1e-3,), **kw)
    ocfg, params, ids, gp, ctx = _setup(zo, torch, arch, 1, B, S, a_bits=a_bits, **kw)
    ctx.zo_forward_quant(to_dev(ids, torch), None, B, S, seed=9, eps_signed=1e-3)
    assert ctx.zo_debug_routes() & zo.ROUTE_GEMM_SPLIT_K
    # both branches of a step in one launch: (branch, range) pairs share the grid's third dimension
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=100, eps=1e-3, lr=1e-3).cpu().numpy()
    assert ctx.zo_debug_routes() & zo.ROUTE_GEMM_SPLIT_K
    for branch, sign in ((0, 1.0), (1, -1.0)):           # the residual stream each branch left behind
        trace = {}
        ref = orc.forward(ocfg, params, ids=ids, seed=100, eps_signed=np.float32(sign * 1e-3), trace=trace)
        assert abs(out[branch] - ref) <= 1e-3 * abs(ref), (branch, out, ref)
        x = ctx.zo_debug_buffer(2, branch).view(torch.bfloat16).float().cpu().numpy().reshape(B * S, -1)
        assert _row_rel(x, trace["l0.out"]).max() < 1e-2
    ctx.close()


@pytest.mark.parametrize("arch", ["llama", "opt"])
@pytest.mark.parametrize("a_bits", [16, 8])
def test_zo_step_fp32_mode(arch, a_bits):
    torch, zo = gpu()
    B, S = 2, 24
    ocfg, params, ids, gp, ctx = _setup(zo, torch, arch, 0, B, S, a_bits=a_bits)
    idd = to_dev(ids, torch)
    eps, lr = 1e-3, 1e-3
    for step in range(3):
        before = [p.copy() for p in params]
        out = ctx.zo_step(idd, None, B, S, seed=100 + step, eps=eps, lr=lr).cpu().numpy()
        lp, lm, g = orc.zo_step(ocfg, params, 100 + step, eps, lr, ids=ids)
        assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm)
        # fp32 storage of a loss ~6.5 resolves 4.8e-7, i.e. 2.4e-4 in g; with activation codes a
        # rounding tie (see _clean_rows) moves one token's loss by ~1e-3 / (B S)
        if a_bits == 16:
            assert abs(out[2] - g) <= 1e-3 * abs(g) + 1e-3, (out[2], g)
        else:
            # one flipped code changes a loss by ~1e-3 / (B S); the quotient divides that by 2 eps
            assert abs(out[2] - g) <= 0.25 * abs(g) + 1.0, (out[2], g)
        assert out[3] == np.float32(np.float64(np.float32(lr)) * np.float64(out[2]))
        # the update itself is bit-exact given the coefficient the GPU used
        for i, p0 in enumerate(before):
            want = orc.update(p0.copy(), 100 + step, i, np.float32(out[3]))
            assert np.array_equal(gp[i].cpu().numpy().view(np.uint32), want.view(np.uint32)), i
        # continue both sides from the GPU's weights so that later steps compare like with like
        params[:] = [t.cpu().numpy() for t in gp]
    ctx.close()


def test_zo_step_bf16_mode_losses_and_g_noise():
    torch, zo = gpu()
    B, S = 2, 32
    ocfg, params, ids, gp, ctx = _setup(zo, torch, "llama", 1, B, S)
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=5, eps=1e-3, lr=1e-3).cpu().numpy()
    lp, lm, g = orc.zo_step(ocfg, params, 5, 1e-3, 1e-3, ids=ids)
    assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm)
    # a storage rounding that falls on the other side of a tie moves a loss by ~1e-4 relative
    # (see test_forward_loss_and_layer_outputs); the difference quotient divides that by 2 eps.
    # g itself is exactly the quotient of the two GPU losses (test_step_equals_two_forwards_plus_update).
    assert abs(out[2] - g) <= 2e-4 * abs(lp) / (2 * 1e-3), (out[2], g)
    ctx.close()


def test_step_equals_two_forwards_plus_update():
    torch, zo = gpu()
    B, S = 2, 16
    ocfg, params, ids, gp, ctx = _setup(zo, torch, "opt", 0, B, S)
    idd = to_dev(ids, torch)
    lp = ctx.zo_forward_quant(idd, None, B, S, 7, 1e-3).item()
    lm = ctx.zo_forward_quant(idd, None, B, S, 7, -1e-3).item()
    out = ctx.zo_step(idd, None, B, S, 7, 1e-3, 1e-2).cpu().numpy()
    assert out[0] == np.float32(lp) and out[1] == np.float32(lm)
    assert out[2] == orc.projected_grad(np.float32(lp), np.float32(lm), np.float32(1e-3))
    ctx.close()


def test_lightweight_updates_only_trainable_tensors():
    torch, zo = gpu()
    B, S = 2, 16
    base = dict(n_layers=2, d_model=128, n_heads=4, d_ffn=256, vocab=512, max_seq=S, w_bits=4, w_group=64, a_bits=4)
    ocfg = orc.Config(1, act_dtype=0, lightweight=1, **base)
    cfg = zo.make_config(1, act_dtype=0, lightweight=1, **base)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 63)
    trainable = [n.endswith(".wq") or n.endswith(".wv") for n, _, _ in shapes]
    ids = synth.token_ids(B, S, 512, 64)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S, trainable=trainable)
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=8, eps=1e-3, lr=1e-2).cpu().numpy()
    before = [p.copy() for p in params]
    lp, lm, g = orc.zo_step(ocfg, params, 8, 1e-3, 1e-2, ids=ids, trainable=trainable)
    assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[2] - g) <= 1e-3 * abs(g) + 2e-3
    for i, p0 in enumerate(before):
        got = gp[i].cpu().numpy()
        if trainable[i]:
            assert np.array_equal(got, orc.update(p0.copy(), 8, i, np.float32(out[3])))
        else:
            assert np.array_equal(got, p0)
    ctx.close()


def test_single_linear_config_one_spsa_step():
    # in = out = 256, W4 g64 asymmetric, A8 per-token, 8 tokens, MSE, eps 1e-3, eta 1e-4, seed 0
    torch, zo = gpu()
    ocfg = orc.Config(0, d_model=256, d_ffn=256, w_bits=4, w_group=64, a_bits=8, act_dtype=0)
    cfg = zo.make_config(0, d_model=256, d_ffn=256, w_bits=4, w_group=64, a_bits=8, act_dtype=0)
    W = synth.weights((256, 256), 65)
    x = synth.activations((8, 256), 66)
    tgt = synth.activations((8, 256), 67)
    gw = to_dev(W, torch)
    ctx = zo.Context(cfg, [gw], 8, 1)
    out = ctx.zo_step(to_dev(x, torch), to_dev(tgt, torch), 8, 1, seed=0, eps=1e-3, lr=1e-4).cpu().numpy()
    y = ctx.zo_debug_buffer(1, 0).view(torch.float32).cpu().numpy().reshape(8, 256)
    trace = {}
    orc.forward(ocfg, [W], x=x, target=tgt, seed=0, eps_signed=np.float32(1e-3), trace=trace)
    assert rel_l2(y, trace["y"]) < 1e-4
    W0 = W.copy()
    lp, lm, g = orc.zo_step(ocfg, [W], 0, 1e-3, 1e-4, x=x, target=tgt)
    assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm)
    assert abs(out[2] - g) <= 1e-3 * abs(g) + 1e-4
    assert np.array_equal(gw.cpu().numpy(), orc.update(W0, 0, 0, np.float32(out[3])))
    ctx.close()


def test_bad_arguments_are_reported_not_launched():
    torch, zo = gpu()
    B, S = 2, 16
    ocfg, params, ids, gp, ctx = _setup(zo, torch, "llama", 0, B, S)
    idd = to_dev(ids, torch)
    with pytest.raises(zo.ZoError) as e:
        ctx.zo_forward_quant(idd, None, B, S + 1, 1, 0.0)
    assert e.value.status in (2, 6)
    with pytest.raises(zo.ZoError) as e:
        ctx.zo_step(idd, None, B, S, 1, 0.0, 1e-3)
    assert e.value.status == 1
    with pytest.raises(zo.ZoError):
        zo.Context(zo.make_config(1, n_layers=1, d_model=100, n_heads=4, d_ffn=256, vocab=64, max_seq=16), gp, B, S)
    ctx.close()


@pytest.mark.parametrize("heads,S", [(2, 40), (1, 200), (2, 128), (1, 257)])
def test_matrix_core_attention_path(heads, S):
    # bf16 storage with head dimension 64 / 128 runs the matrix-core attention kernel; S spans
    # several key tiles, a ragged last query tile and a ragged last key tile
    torch, zo = gpu()
    B = 2
    ocfg, params, ids, gp, ctx = _setup(zo, torch, "llama", 1, B, S, n_layers=1, n_heads=heads, a_bits=16)
    idd = to_dev(ids, torch)
    loss = ctx.zo_forward_quant(idd, None, B, S, seed=4, eps_signed=1e-3).item()
    trace = {}
    ref = orc.forward(ocfg, params, ids=ids, seed=4, eps_signed=np.float32(1e-3), trace=trace)
    assert abs(loss - ref) <= 1e-3 * abs(ref), (loss, ref)
    x = ctx.zo_debug_buffer(2).view(torch.bfloat16).float().cpu().numpy().reshape(B * S, -1)
    # the probabilities enter the second product as bf16 operands (see test_gpu_attention.py):
    # whole-tensor error within the bf16 tolerance, single rows within twice that
    assert rel_l2(x, trace["l0.out"]) < 1e-2
    assert _row_rel(x, trace["l0.out"]).max() < 2e-2
    ctx.close()


def test_profile_mask_brackets_only_the_selected_categories():
    """Per-launch timing restricted to one category: the others report no bracketed group, the selected one the same
    launch count as the unrestricted session."""
    torch, zo = gpu()
    B, S = 2, 80                                               # 160 tokens: the quantize-once route, batched GEMMs
    ocfg, params, ids, gp, ctx = _setup(zo, torch, "llama", 1, B, S)
    idd = to_dev(ids, torch)
    ctx.zo_profile_begin()
    ctx.zo_step(idd, None, B, S, seed=3, eps=1e-3, lr=0.0)
    full = ctx.zo_profile_end()
    ctx.zo_profile_begin_mask(("gemm",))
    ctx.zo_step(idd, None, B, S, seed=3, eps=1e-3, lr=0.0)
    only = ctx.zo_profile_end()
    assert only["gemm"][1] == full["gemm"][1] > 0 and only["gemm"][0] > 0.0
    assert all(only[k][1] == 0 for k in only if k != "gemm")
    assert full["weight_quant"][1] > 0 and full["update"][1] > 0
    ctx.close()
