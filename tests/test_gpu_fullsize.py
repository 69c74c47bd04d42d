"""GPU parity at the full sizes of the benchmark workload (Llama-2-7B shape, 8 x 1024 tokens), in
the launch configurations bench.py times.  The weight quantizer and the update are compared with
the oracle on whole 45 M-parameter tensors; the GEMM and attention on sampled outputs that the
oracle computes one by one; the whole 7B step through properties that hold at any size.  Inputs
are seeded and synthetic (weights 0.02 N(0,1), activations N(0,1), uniform token ids)."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu

M, D, F = 8192, 4096, 11008


def test_weight_quant_full_matrix():
    torch, zo = gpu()
    W = synth.weights((F, D), 81)                      # w_gate / w_up shape, 45 M parameters
    eps = np.float32(1e-3)
    out = zo.zo_debug_quant_weight(to_dev(W, torch), 4, 64, seed=3, tensor_id=7, eps_signed=float(eps), out_dtype=1)
    ref = orc.fakequant_weight(W, 4, 64, 3, 7, eps, round_bf16=True)        # the whole matrix: a few seconds on the host
    assert np.array_equal(out["step"].cpu().numpy().view(np.uint32), ref["step"].view(np.uint32))
    assert np.array_equal(out["zp"].cpu().numpy(), ref["zp"])
    codes = out["codes"].cpu().numpy()
    assert int(np.sum(codes != ref["codes"].astype(np.uint8))) == 0
    what = out["what"].float().cpu().numpy()
    assert int(np.sum(what.view(np.uint32) != ref["what"].view(np.uint32))) == 0


def test_update_full_tensor():
    torch, zo = gpu()
    n = F * D
    w = synth.weights((n,), 82)
    g = to_dev(w, torch)
    c = np.float32(2.5e-4)
    zo.zo_update_tensor(g, seed=11, tensor_id=5, coeff_host=float(c))
    want = orc.update(w.copy(), 11, 5, c)
    assert np.array_equal(g.cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("N,K", [(3 * D, D), (D, F)])
def test_gemm_full_shape_sampled_outputs(N, K):
    torch, zo = gpu()
    X = orc.bf16_round(synth.activations((M, K), 83))
    W = orc.bf16_round(synth.weights((N, K), 84))
    Y = zo.zo_gemm_nt(to_dev(X, torch, torch.bfloat16), to_dev(W, torch, torch.bfloat16))
    rng = synth.rng(85)
    ms = np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 60)])
    ns = np.concatenate([[0, 255, 256, N - 1], rng.integers(0, N, 60)])
    got = Y[torch.from_numpy(ms).cuda()][:, torch.from_numpy(ns).cuda()].float().cpu().numpy()
    ref = X[ms].astype(np.float64) @ W[ns].astype(np.float64).T
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * np.sqrt(K))


def test_gate_up_gemm_with_swiglu_full_shape_sampled_outputs():
    """The 8192 x 22016 x 4096 gate | up GEMM of the benchmark with SwiGLU in its epilogue (rows interleaved in blocks of
    32 channels): sampled (token, channel) outputs against the definition with the same rounding points."""
    torch, zo = gpu()
    X = orc.bf16_round(synth.activations((M, D), 87))
    G = orc.bf16_round(synth.weights((F, D), 88, scale=0.3))
    U = orc.bf16_round(synth.weights((F, D), 89, scale=0.3))
    Wi = np.stack([G.reshape(F // 32, 32, D), U.reshape(F // 32, 32, D)], axis=1).reshape(2 * F, D)
    Y = zo.zo_gemm_nt_swiglu(to_dev(X, torch, torch.bfloat16), to_dev(Wi, torch, torch.bfloat16))
    rng = synth.rng(90)
    ms = np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 60)])
    cs = np.concatenate([[0, 31, 32, 127, 128, F - 1], rng.integers(0, F, 58)])
    got = Y[torch.from_numpy(ms).cuda()][:, torch.from_numpy(cs).cuda()].float().cpu().numpy()
    g = orc.bf16_round((X[ms].astype(np.float64) @ G[cs].astype(np.float64).T).astype(np.float32)).astype(np.float64)
    u = orc.bf16_round((X[ms].astype(np.float64) @ U[cs].astype(np.float64).T).astype(np.float32)).astype(np.float64)
    ref = g / (1.0 + np.exp(-g)) * u
    # one bf16 rounding of the product; gate / up may round to the neighbouring bf16 value (fp32 against fp64 sums)
    assert np.mean(np.abs(got - ref) > 2.0 ** -8 * np.abs(ref) + 1e-6) < 3e-2
    assert np.all(np.abs(got - ref) <= 2.0 ** -6 * np.abs(ref) + 2e-2)


@pytest.mark.parametrize("group", [0, 64])
def test_integer_route_linear_full_shape_sampled_outputs(group):
    """One quantized linear of the benchmark's q | k | v shape (8192 x 12288 x 4096, W4A8) on the integer route -- per-channel
    steps (integer accumulation over all of K inside the matrix unit) and groups of 64 (rescale per slice) -- at eps = 0, so
    that sampled rows of W quantize as they do inside the whole matrix: sampled outputs against the un-rounded operand
    product of the oracle's codes."""
    torch, zo = gpu()
    N, K = 12288, 4096
    X = orc.bf16_round(synth.activations((M, K), 95))
    W = synth.weights((N, K), 96)
    Y = zo.zo_linear_fakequant_mma(to_dev(X, torch, torch.bfloat16), to_dev(W, torch), 4, group, 8, 0, 0, 0.0, out_f32=True)
    rng = synth.rng(97)
    ms = np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 28)])
    ns = np.concatenate([[0, 255, 256, N - 1], rng.integers(0, N, 28)])
    qa = orc.fakequant_act(X[ms], 8, False)
    qw = orc.fakequant_weight(W[ns], 4, group, eps_signed=0.0)
    ref = qa["xhat"].astype(np.float64) @ qw["what"].astype(np.float64).T
    mag = np.abs(qa["xhat"].astype(np.float64)) @ np.abs(qw["what"].astype(np.float64)).T
    got = Y[torch.from_numpy(ms).cuda()][:, torch.from_numpy(ns).cuda()].cpu().numpy()
    assert np.all(np.abs(got - ref) <= 4e-6 * mag + 1e-30), (np.abs(got - ref) / mag).max()


def test_lm_head_loss_full_shape_sampled_rows():
    """The 8192 x 32000 x 4096 lm_head GEMM of the benchmark with the cross entropy in its epilogue: sampled row losses
    against the definition in fp64 (logits of a row: 32000 dot products the host computes one row at a time)."""
    torch, zo = gpu()
    V, S = 32000, 1024
    X = orc.bf16_round(synth.activations((M, D), 91) * 0.5)
    W = orc.bf16_round(synth.weights((V, D), 92, scale=0.05))
    ids = synth.token_ids(M // S, S, V, 93).reshape(-1).astype(np.int32)
    got = zo.zo_gemm_nt_ce(to_dev(X, torch, torch.bfloat16), to_dev(W, torch, torch.bfloat16), to_dev(ids, torch), S).cpu().numpy()
    assert np.array_equal(got[S - 1::S], np.zeros(M // S, np.float32))
    rng = synth.rng(94)
    W64 = W.astype(np.float64)
    for m in np.concatenate([[0, 255, 256, M - 2], rng.integers(0, M, 12)]):
        if m % S == S - 1:
            continue
        lg = W64 @ X[m].astype(np.float64)
        ref = np.log(np.exp(lg - lg.max()).sum()) + lg.max() - lg[ids[m + 1]]
        assert abs(got[m] - ref) <= 2e-5 * (np.abs(lg).max() + np.log(V)) + 1e-5, (m, got[m], ref)


def test_attention_full_shape_sampled_heads():
    torch, zo = gpu()
    B, S, H, dh = 8, 1024, 32, 128
    qkv = orc.bf16_round(synth.activations((B * S, 3 * H * dh), 86))
    out = zo.zo_attention_causal(to_dev(qkv, torch, torch.bfloat16), B, S, H, dh).float().cpu().numpy()
    d = H * dh
    for b, h in ((0, 0), (3, 17), (7, 31)):
        rows = slice(b * S, (b + 1) * S)
        cols = slice(h * dh, (h + 1) * dh)
        sub = np.concatenate([qkv[rows, cols], qkv[rows, d + h * dh:d + (h + 1) * dh], qkv[rows, 2 * d + h * dh:2 * d + (h + 1) * dh]], 1)
        ref = orc._attention(sub[:, :dh], sub[:, dh:2 * dh], sub[:, 2 * dh:], 1, S, 1, dh)
        got = out[rows, cols]
        err = np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)
        assert err.max() < 8e-3, (b, h, err.max())


def test_full_7b_step_properties():
    """One zo_step of the benchmark workload itself (6.74 B parameters, W4A8 g64, 8 x 1024 tokens)."""
    torch, zo = gpu()
    cfg = zo.make_config(zo.ARCH_LLAMA, n_layers=32, d_model=D, n_heads=32, d_ffn=F, vocab=32000, max_seq=1024,
                         w_bits=4, w_group=64, a_bits=8, act_dtype=zo.ACT_BF16)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    params = []
    for i in range(zo.zo_num_params(cfg)):
        n = zo.zo_param_numel(cfg, i)
        t = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=gen)
        if n == D:
            t.add_(1.0)
        params.append(t)
    ids = torch.randint(0, 32000, (8, 1024), dtype=torch.int32, device="cuda", generator=gen)
    probe = [0, 2, 7, 9, 100, len(params) - 2, len(params) - 1]      # embedding, wq, w_gate, w_down, a gain, final norm, lm_head
    before = {i: params[i].cpu().numpy() for i in probe}
    ctx = zo.Context(cfg, params, 8, 1024)
    eps, lr, seed = 1e-3, 1e-4, 42
    out = ctx.zo_step(ids, None, 8, 1024, seed=seed, eps=eps, lr=lr).cpu().numpy()
    lp, lm, g, c = (np.float32(v) for v in out)
    assert np.isfinite(out).all()
    # random-init losses sit near ln(vocab) (plus half the logit variance)
    assert 10.0 < lp < 12.5 and 10.0 < lm < 12.5 and lp != lm
    assert g == orc.projected_grad(lp, lm, np.float32(eps))                      # Eq. 2, q = 1
    assert c == orc.coeff(np.float32(lr), g)
    for i in probe:                                                              # Eq. 3 on whole tensors, bit-exact
        want = orc.update(before[i].copy(), seed, i, c)
        assert np.array_equal(params[i].cpu().numpy().view(np.uint32), want.view(np.uint32)), i
    # the same seed and batch again from the updated weights: a different loss pair (weights moved)
    out2 = ctx.zo_step(ids, None, 8, 1024, seed=seed, eps=eps, lr=0.0).cpu().numpy()
    assert out2[0] != out[0] and abs(out2[0] - out[0]) < 0.05
    # and a zero learning rate leaves the weights untouched
    assert np.array_equal(params[2].cpu().numpy(), orc.update(before[2].copy(), seed, 2, c))
    ctx.close()
