"""Model-level GPU parity at the widths of the benchmark workloads: one decoder layer of the real width (all of
d_model, heads, d_ffn and the vocabulary), one sequence, bf16 storage, both forwards of Eq. 2 through zo_step against
the oracle's zo_step on the same seeded inputs -- the compositions bench.py times (kernel selection depends on the
widths and the token count: loss formed in the lm_head GEMM, SwiGLU / rotary embedding in GEMM epilogues, 256-row GEMM
tiles, the one-workgroup-per-row norm + quantizer), not only their parts.  The last test is the tiny decoder
configuration exactly, ten consecutive steps.  Tolerances: losses 1e-3 relative (the benchmark spec); g is exactly the
quotient of the device losses and is reported against the oracle's (bf16 storage: see test_gpu_g_parity.py);
updated masters bit-exact given the device's coefficient."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu

EPS = 1e-3


def _row_rel(a, b):
    return np.linalg.norm(a.astype(np.float64) - b, axis=1) / np.maximum(np.linalg.norm(b, axis=1), 1e-30)


def _one_layer_step(arch, S, routes_want, lightweight=0, lr=1e-3, loss_tol=1e-3, mma=0, **kw):
    torch, zo = gpu()
    base = dict(n_layers=1, max_seq=S, **kw)
    ocfg = orc.Config(arch, act_dtype=1, lightweight=lightweight, mma=mma, **base)
    cfg = zo.make_config(arch, act_dtype=1, lightweight=lightweight, mma=mma, **base)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 1234)
    ids = synth.token_ids(1, S, kw["vocab"], 5678)
    trainable = None
    o_params, g_params = list(params), [to_dev(p, torch) for p in params]
    if lightweight:
        trainable = [n.endswith(".wq") or n.endswith(".wv") for n, _, _ in shapes]
        for i, (w, t, (_, _, q)) in enumerate(zip(params, trainable, shapes)):
            if q and not t:
                o_params[i] = orc.pack_int4(w, kw["w_group"])
                g_params[i] = zo.zo_pack_weight_int4(g_params[i], kw["w_group"])
    ctx = zo.Context(cfg, g_params, 1, S, trainable=trainable)
    out = ctx.zo_step(to_dev(ids, torch), None, 1, S, seed=0, eps=EPS, lr=lr).cpu().numpy()
    routes = ctx.zo_debug_routes()
    # the oracle's step, taken apart so that both forwards leave their stored activations behind: Eq. 2's two losses,
    # the projected gradient, the coefficient, and (below) Eq. 3 on the tensors that are compared
    ref_loss = []
    for branch, sign in ((0, 1.0), (1, -1.0)):
        trace = {}
        ref_loss.append(orc.forward(ocfg, o_params, ids=ids, seed=0, eps_signed=np.float32(sign * EPS), trainable=trainable, trace=trace))
        # q | k | v lie upstream of everything that amplifies rounding noise: one norm + quantizer and one linear away
        # from the embedding.  A row may carry a flipped activation code; almost every row agrees to rounding.
        qkv = ctx.zo_debug_buffer(3, branch).view(torch.bfloat16).float().cpu().numpy().reshape(S, -1)
        err = _row_rel(qkv, trace["l0.qkv"])
        assert np.median(err) < 1e-4 and np.quantile(err, 0.9) < 1e-3 and err.max() < 5e-2, (branch, np.median(err), err.max())
        attn = ctx.zo_debug_buffer(4, branch).view(torch.bfloat16).float().cpu().numpy().reshape(S, -1)
        err = _row_rel(attn, trace["l0.attn"])
        assert np.median(err) < 5e-3 and err.max() < 3e-2, (branch, np.median(err), err.max())
        x = ctx.zo_debug_buffer(2, branch).view(torch.bfloat16).float().cpu().numpy().reshape(S, -1)
        e_out = np.linalg.norm(x - trace["l0.out"]) / np.linalg.norm(trace["l0.out"])
        print("branch %d: layer output, whole tensor relative l2 error %.2e" % (branch, e_out))
        if kw["a_bits"] == 16:
            assert e_out < 1e-2
    lp, lm = ref_loss
    g = orc.projected_grad(lp, lm, np.float32(EPS))
    print("gpu L+ %.6f L- %.6f g %+.4f | oracle L+ %.6f L- %.6f g %+.4f | routes 0x%x" % (out[0], out[1], out[2], lp, lm, g, routes))
    assert abs(out[0] - lp) <= loss_tol * abs(lp) and abs(out[1] - lm) <= loss_tol * abs(lm)
    assert out[2] == orc.projected_grad(np.float32(out[0]), np.float32(out[1]), np.float32(EPS))
    assert out[3] == orc.coeff(np.float32(lr), out[2])
    assert routes & ~zo.ROUTE_GEMM_SPLIT_K == routes_want, hex(routes)      # a K split of narrow GEMMs is a launch detail
    # Eq. 3 on the first quantized linear and on the lm_head, bit-exact given the device's coefficient
    for i in (2, len(shapes) - 1):
        if trainable is not None and not trainable[i]:
            if isinstance(o_params[i], np.ndarray):
                assert np.array_equal(g_params[i].cpu().numpy(), o_params[i])
            continue
        assert np.array_equal(g_params[i].cpu().numpy(), orc.update(o_params[i].copy(), 0, i, np.float32(out[3])))
    ctx.close()


@pytest.mark.parametrize("w_bits,a_bits", [(4, 8), (2, 16)])
def test_llama7b_widths_one_layer(w_bits, a_bits):
    torch, zo = gpu()
    _one_layer_step(1, 1024, zo.ROUTE_SWIGLU_IN_GEMM | zo.ROUTE_ROPE_IN_GEMM | zo.ROUTE_CE_IN_GEMM,
                    d_model=4096, n_heads=32, d_ffn=11008, vocab=32000, w_bits=w_bits, w_group=64, a_bits=a_bits)


@pytest.mark.parametrize("mma", [0, 1])
def test_llama7b_widths_one_layer_per_channel(mma):
    """Per-channel weight steps (the weight setting of the W4A4 rows of the appendix's quantization settings) at the 7B widths:
    through the bf16 contraction (row quantizer with interleaved outputs, all three GEMM epilogues) and through the integer
    route (codes, integer accumulation over all of K, SwiGLU in the integer GEMM's epilogue, stand-alone rotary kernel)."""
    torch, zo = gpu()
    routes = zo.ROUTE_SWIGLU_IN_GEMM | zo.ROUTE_CE_IN_GEMM | (zo.ROUTE_INT8_MMA if mma else zo.ROUTE_ROPE_IN_GEMM)
    _one_layer_step(1, 1024, routes, mma=mma, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000, w_bits=4, w_group=0, a_bits=8)


def test_opt1p3b_widths_one_layer():
    """64-wide heads, LayerNorm, biases, ReLU, and a vocabulary (50272 = 2^5 * 1571) that ends inside a GEMM tile on
    the loss-in-GEMM route."""
    torch, zo = gpu()
    _one_layer_step(2, 512, zo.ROUTE_CE_IN_GEMM, d_model=2048, n_heads=32, d_ffn=8192, vocab=50272, w_bits=4, w_group=128, a_bits=8)


@pytest.mark.parametrize("a_bits", [8, 4])
def test_llama13b_lightweight_widths_one_layer(a_bits):
    """Frozen linears as packed 4-bit codes (group 128), trainable query / value projections.  With 8-bit activations the
    losses hold the 1e-3 of the other workloads.  With the configuration's 4-bit per-token activations they cannot: a
    code step is half a standard deviation of its row (15 steps over ~8 sigma), so an input disagreement of relative size
    e flips a fraction ~2e of the codes by a whole step and comes out as ~sqrt(e / 2): the 2.5e-3 per row that the bf16
    probabilities of the matrix-core attention add (see test_gpu_attention.py) grow to 3.5e-2 after the attention-output
    quantizer, 0.13 after the FFN's, ~0.3 after the down projection's -- in the oracle's arithmetic just as on the GPU,
    whichever of two valid roundings a side takes.  Token losses then differ by O(0.3) each way and their mean over
    1023 positions by ~1e-2 = 1e-3 relative: the bound asserted here is 3e-3, and what lies upstream of the attention
    (q | k | v) and the attention itself are held as sharply as in every other configuration."""
    torch, zo = gpu()
    _one_layer_step(1, 1024, zo.ROUTE_SWIGLU_IN_GEMM | zo.ROUTE_ROPE_IN_GEMM | zo.ROUTE_CE_IN_GEMM, lightweight=1,
                    loss_tol=1e-3 if a_bits == 8 else 3e-3,
                    d_model=5120, n_heads=40, d_ffn=13824, vocab=32000, w_bits=4, w_group=128, a_bits=a_bits)


def test_tiny_decoder_ten_steps():
    """The tiny decoder configuration as given: 4 layers, d 512, 8 heads, SwiGLU 2048, RMSNorm, vocabulary 4096, W4A16
    group 64, 8 x 128 uniform-random ids, bf16 activations, 10 ZO steps.  After every step both sides continue from the
    GPU's masters (g in bf16 storage carries rounding noise, so the trajectories would otherwise drift apart by design)."""
    torch, zo = gpu()
    B, S = 8, 128
    base = dict(n_layers=4, d_model=512, n_heads=8, d_ffn=2048, vocab=4096, max_seq=S, w_bits=4, w_group=64, a_bits=16)
    ocfg = orc.Config(1, act_dtype=1, **base)
    cfg = zo.make_config(1, act_dtype=1, **base)
    params = synth.model_params(orc.param_shapes(ocfg), 1234)
    gp = [to_dev(p, torch) for p in params]
    ctx = zo.Context(cfg, gp, B, S)
    lr = 1e-4
    dgs = []
    for step in range(10):
        ids = synth.token_ids(B, S, base["vocab"], 5678 + step)
        before = [p.copy() for p in params]
        out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=step, eps=EPS, lr=lr).cpu().numpy()
        lp, lm, g = orc.zo_step(ocfg, params, step, EPS, lr, ids=ids)
        assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm), (step, out, lp, lm)
        assert out[2] == orc.projected_grad(np.float32(out[0]), np.float32(out[1]), np.float32(EPS))
        dgs.append(float(out[2]) - float(g))
        for i in (0, 2, 8, len(params) - 1):
            assert np.array_equal(gp[i].cpu().numpy(), orc.update(before[i].copy(), step, i, np.float32(out[3]))), (step, i)
        params[:] = [t.cpu().numpy() for t in gp]
    print("tiny decoder, 10 steps: delta g (gpu - oracle) " + " ".join("%+.3f" % v for v in dgs))
    ctx.close()
