"""GPU parity of the lm_head GEMM with the cross entropy in its epilogue (the loss L of Eq. 2 on a decoder; the logits
are never stored) against the definition written out in fp64 on the same bf16 operands, and of a decoder forward that
takes this route against the oracle's forward."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


def _row_losses(X, W, ids, S):
    lg = X.astype(np.float64) @ W.astype(np.float64).T
    N = W.shape[0]
    mx = lg.max(1)
    lse = np.log(np.exp(lg - mx[:, None]).sum(1)) + mx
    tgt = np.clip(np.roll(ids, -1), 0, N - 1)
    out = lse - lg[np.arange(len(ids)), tgt]
    out[S - 1::S] = 0.0
    return out, lg


@pytest.mark.parametrize("B,S,N,K,scale", [(4, 256, 8192, 128, 1.0), (4, 250, 8400, 64, 1.0), (2, 600, 7050, 192, 8.0),
                                           (32, 64, 4100, 64, 1.0)])
def test_ce_epilogue_matches_definition(B, S, N, K, scale):
    """Ragged M (1000 and 1200 rows: the last m-tile is partly filled), vocabularies that end inside a wave's 64 columns
    and inside a lane's group of four, sharp logits (scale 8: the per-tile maxima differ by tens of units)."""
    torch, zo = gpu()
    M = B * S
    X = orc.bf16_round(synth.activations((M, K), 141) * scale)
    W = orc.bf16_round(synth.weights((N, K), 142, scale=0.3))
    ids = synth.token_ids(B, S, N, 143).reshape(-1).astype(np.int32)
    ids[5], ids[77], ids[M - 3] = -4, N + 9, N - 1                       # out-of-range ids clamp to the vocabulary's ends
    ids[S + 1], ids[3] = 0, N - (N % 256 or 256)                         # first column, first column of the last tile
    got = zo.zo_gemm_nt_ce(to_dev(X, torch, torch.bfloat16), to_dev(W, torch, torch.bfloat16), to_dev(ids, torch), S).cpu().numpy()
    ref, lg = _row_losses(X, W, ids, S)
    assert np.array_equal(got[S - 1::S], np.zeros(B, np.float32))
    # fp32 accumulation of K products per logit, fp32 exponentials and sums: absolute error of a row loss
    tol = 2e-5 * (np.abs(lg).max(1) + np.log(N)) + 1e-5
    assert np.all(np.abs(got - ref) <= tol), np.abs(got - ref).max()
    # the mean is the oracle's cross entropy of the same logits
    mean = got.reshape(B, S)[:, :-1].mean()
    ids_c = np.clip(ids, 0, N - 1).reshape(B, S)
    assert abs(mean - orc.cross_entropy(lg, ids_c, B, S)) <= 1e-5 * abs(mean) + 1e-6


def test_ce_gemm_rejects_small_or_odd_shapes():
    torch, zo = gpu()
    X = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((128, 64), dtype=torch.bfloat16, device="cuda")
    ids = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(zo.ZoError) as e:
        zo.zo_gemm_nt_ce(X, W, ids, 16)
    assert e.value.status == 5
    X = torch.zeros((4096, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((4096, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(zo.ZoError) as e:
        zo.zo_gemm_nt_ce(X, W, torch.zeros(4096, dtype=torch.int32, device="cuda"), 100)     # S does not divide M
    assert e.value.status == 2


@pytest.mark.parametrize("arch", ["llama", "opt"])
def test_decoder_step_with_ce_in_the_gemm(arch):
    """1024 tokens, vocabulary 8192: the lm_head is large enough for the route.  Both losses against the oracle, the
    route flag, and no logits to hand out afterwards."""
    torch, zo = gpu()
    kw = dict(n_layers=1, d_model=128, n_heads=2, d_ffn=256, vocab=8192, max_seq=256, w_bits=4, w_group=64, a_bits=8)
    B, S = 4, 256
    oarch, zarch = (orc.ARCH_LLAMA, zo.ARCH_LLAMA) if arch == "llama" else (orc.ARCH_OPT, zo.ARCH_OPT)
    ocfg = orc.Config(oarch, act_dtype=1, **kw)
    params = synth.model_params(orc.param_shapes(ocfg), 144)
    params = [p * (3.0 if p.ndim == 2 else 1.0) for p in params]
    ids = synth.token_ids(B, S, kw["vocab"], 145)
    lp, lm, g = orc.zo_step(ocfg, [p.copy() for p in params], 21, 1e-3, 0.0, ids=ids)
    ctx = zo.Context(zo.make_config(zarch, act_dtype=zo.ACT_BF16, **kw), [to_dev(p, torch) for p in params], B, S)
    out = ctx.zo_step(to_dev(ids, torch), None, B, S, seed=21, eps=1e-3, lr=0.0).cpu().numpy()
    assert ctx.zo_debug_routes() & zo.ROUTE_CE_IN_GEMM
    assert abs(out[0] - lp) <= 1e-3 * abs(lp) and abs(out[1] - lm) <= 1e-3 * abs(lm), (out, lp, lm)
    with pytest.raises(zo.ZoError) as e:
        ctx.zo_debug_buffer(1)
    assert e.value.status == 5
    # a single forward (one branch per launch) takes the same route and gives the step's losses bit for bit (lr was 0)
    for sign, want in ((1.0, out[0]), (-1.0, out[1])):
        got = ctx.zo_forward_quant(to_dev(ids, torch), None, B, S, seed=21, eps_signed=sign * 1e-3).item()
        assert ctx.zo_debug_routes() & zo.ROUTE_CE_IN_GEMM
        assert np.float32(got) == np.float32(want), (got, want)
    ctx.close()
