"""GPU parity of the gate / up GEMM with SwiGLU in its epilogue (gate and up rows interleaved in blocks of 32 channels)
against the oracle's GEMM + SwiGLU with the same rounding points, and of a Llama-shaped step that takes this route."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev, rel_l2

pytestmark = pytest.mark.gpu


def _interleave(gate, up):
    f, K = gate.shape
    return np.stack([gate.reshape(f // 32, 32, K), up.reshape(f // 32, 32, K)], axis=1).reshape(2 * f, K)


@pytest.mark.parametrize("M,f,K", [(2048, 2048, 256), (2100, 2080, 128), (4096, 1056, 64)])
def test_swiglu_epilogue_matches_gemm_then_swiglu(M, f, K):
    """Ragged M and a last n-tile that is only partly filled (2 f not a multiple of 256)."""
    torch, zo = gpu()
    X = orc.bf16_round(synth.activations((M, K), 131))
    G = orc.bf16_round(synth.weights((f, K), 132, scale=0.3))
    U = orc.bf16_round(synth.weights((f, K), 133, scale=0.3))
    Y = zo.zo_gemm_nt_swiglu(to_dev(X, torch, torch.bfloat16), to_dev(_interleave(G, U), torch, torch.bfloat16)).float().cpu().numpy()
    # reference with the same rounding points: gate and up rounded to bf16 as if stored, product rounded once
    g = orc.bf16_round(orc.linear(X, G).astype(np.float32)).astype(np.float64)
    u = orc.bf16_round(orc.linear(X, U).astype(np.float32)).astype(np.float64)
    ref = g / (1.0 + np.exp(-g)) * u
    assert rel_l2(Y, ref) < 4e-3
    # one bf16 rounding of the result, plus gate / up that round to the neighbouring bf16 value when the fp32 sum
    # of K products lands on the other side of a rounding boundary than the fp64 sum
    assert np.mean(np.abs(Y - ref) > 2.0 ** -8 * np.abs(ref) + 1e-6) < 2e-2
    # and against the library's own two-kernel route (plain GEMM, then the same activation on the stored values)
    gu = zo.zo_gemm_nt(to_dev(X, torch, torch.bfloat16), to_dev(np.concatenate([G, U]), torch, torch.bfloat16)).float()
    gg, uu = gu[:, :f], gu[:, f:]
    two = (gg / (1.0 + torch.exp(-gg)) * uu).to(torch.bfloat16).float().cpu().numpy()
    assert np.mean(Y != two) < 2e-2 and np.all(np.abs(Y - two) <= 2.0 ** -7 * np.abs(two) + 1e-6)


def test_swiglu_gemm_rejects_small_or_odd_shapes():
    torch, zo = gpu()
    X = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((128, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(zo.ZoError) as e:
        zo.zo_gemm_nt_swiglu(X, W)
    assert e.value.status == 5


@pytest.mark.parametrize("a_bits,lightweight", [(16, 0), (8, 0), (8, 1)])
def test_llama_step_with_swiglu_in_the_gemm(a_bits, lightweight):
    """1024 tokens, f = 4096: the gate / up GEMM is large enough for the route (one GEMM launch fewer kernels: no
    separate activation pass).  Losses against the oracle and against the route with the separate kernels."""
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=128, n_heads=2, d_ffn=4096, vocab=256, max_seq=256, w_bits=4, w_group=64, a_bits=a_bits)
    B, S = 4, 256
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=1, lightweight=lightweight, **kw)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 134)
    trainable = [n.endswith(".wq") or n.endswith(".wv") for n, _, _ in shapes] if lightweight else None
    ids = synth.token_ids(B, S, 256, 135)
    o_params = [orc.pack_int4(w, 64) if (lightweight and q and not t) else w.copy()
                for w, (_, _, q), t in zip(params, shapes, trainable or [True] * len(shapes))]
    lp = orc.forward(ocfg, o_params, ids=ids, seed=8, eps_signed=1e-3, trainable=trainable)
    outs = []
    for no_fused in (0, 1):
        cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=1, lightweight=lightweight, no_fused=no_fused, **kw)
        gp = [zo.zo_pack_weight_int4(to_dev(w, torch), 64) if (lightweight and q and not t) else to_dev(w, torch)
              for w, (_, _, q), t in zip(params, shapes, trainable or [True] * len(shapes))]
        ctx = zo.Context(cfg, gp, B, S, trainable=trainable)
        ctx.zo_profile_begin()
        out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=8, eps=1e-3, lr=1e-3).cpu().numpy().copy()
        prof = ctx.zo_profile_end()
        assert ctx.zo_debug_routes() & ~zo.ROUTE_GEMM_SPLIT_K == (0 if no_fused else zo.ROUTE_SWIGLU_IN_GEMM)
        outs.append(out)
        assert abs(out[0] - lp) <= 2e-3 * abs(lp)
        ctx.close()
    assert abs(outs[0][0] - outs[1][0]) <= 3e-4 * abs(lp) and abs(outs[0][1] - outs[1][1]) <= 3e-4 * abs(lp)


@pytest.mark.parametrize("a_bits", [16, 8])
def test_llama_step_with_rotary_embedding_in_the_gemm(a_bits):
    """6 x 1024 tokens, 4 heads of 128: the fused q | k | v GEMM is large enough to rotate q and k in its epilogue (head
    blocks permuted in the operand buffer) and the gate / up GEMM to apply SwiGLU.  Loss against the oracle; the final
    hidden state row by row against the route with the stand-alone kernels (same values rounded at the same points)."""
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=512, n_heads=4, d_ffn=1024, vocab=256, max_seq=1024, w_bits=4, w_group=64, a_bits=a_bits)
    B, S = 6, 1024
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=1, **kw)
    params = synth.model_params(orc.param_shapes(ocfg), 141)
    ids = synth.token_ids(B, S, 256, 142)
    ref = orc.forward(ocfg, params, ids=ids, seed=8, eps_signed=1e-3)
    hid, losses = [], []
    for no_fused in (0, 1):
        cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=1, no_fused=no_fused, **kw)
        gp = [to_dev(w, torch) for w in params]
        ctx = zo.Context(cfg, gp, B, S)
        ctx.zo_profile_begin()
        losses.append(ctx.zo_forward_quant(to_dev(ids, torch), None, B, S, seed=8, eps_signed=1e-3).item())
        prof = ctx.zo_profile_end()
        assert ctx.zo_debug_routes() & ~zo.ROUTE_GEMM_SPLIT_K == (0 if no_fused else zo.ROUTE_SWIGLU_IN_GEMM | zo.ROUTE_ROPE_IN_GEMM)
        hid.append(ctx.zo_debug_buffer(0).view(torch.bfloat16).float().cpu().numpy().reshape(B * S, kw["d_model"]).copy())
        assert abs(losses[-1] - ref) <= 1e-3 * abs(ref)
        ctx.close()
    # identical arithmetic up to the order of fp32 sums inside the GEMM tiles: the two routes agree far more closely
    # than either agrees with the fp64 oracle
    assert abs(losses[0] - losses[1]) <= 1e-4 * abs(ref)
    d = np.linalg.norm(hid[0] - hid[1], axis=1) / np.linalg.norm(hid[1], axis=1)
    assert np.median(d) < 2e-3 and d.max() < (3e-2 if a_bits == 16 else 0.2)


def test_rotary_epilogue_moves_q_and_k_only():
    """With eps = 0 and a model whose attention output is read back, permuting head blocks and rotating in the epilogue
    must leave v untouched and give q, k the stand-alone kernel's values: checked through the attention output of a
    one-layer model with identity-like weights being equal on both routes (bit-exact: same bf16 inputs to attention)."""
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=256, n_heads=2, d_ffn=512, vocab=128, max_seq=1024, w_bits=0, w_group=0, a_bits=16)
    B, S = 11, 1024                                         # M * 3 d = 8.65 M: just above the route's threshold
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=1, **kw)
    params = synth.model_params(orc.param_shapes(ocfg), 143)
    ids = to_dev(synth.token_ids(B, S, 128, 144), torch)
    res = []
    for no_fused in (0, 1):
        cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=1, no_fused=no_fused, **kw)
        ctx = zo.Context(cfg, [to_dev(w, torch) for w in params], B, S)
        loss = ctx.zo_forward_quant(ids, None, B, S, seed=1, eps_signed=0.0).item()
        assert ctx.zo_debug_routes() & ~zo.ROUTE_GEMM_SPLIT_K == (0 if no_fused else zo.ROUTE_ROPE_IN_GEMM | zo.ROUTE_SWIGLU_IN_GEMM)
        res.append((loss, ctx.zo_debug_buffer(2).view(torch.bfloat16).float().cpu().numpy().copy()))
        ctx.close()
    assert abs(res[0][0] - res[1][0]) <= 2e-5 * abs(res[1][0])
    diff = np.abs(res[0][1] - res[1][1])
    assert np.mean(diff > 0) < 0.05 and diff.max() <= 2.0 ** -6 * np.abs(res[1][1]).max()
