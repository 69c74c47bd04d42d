"""The K-split GEMM entry point that allocates nothing (its partial sums live in a device array of the library):
against the existing entry point with caller-provided scratch, on two calls in a row, the second with a smaller input
(the array keeps the first call's contents), then a shape that needs no split, then one that exceeds the array."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


def _case(torch, zo, M, N, K, seed, epilogue):
    X = to_dev(orc.bf16_round(synth.activations((M, K), seed)), torch, torch.bfloat16)
    W = to_dev(orc.bf16_round(synth.weights((N, K), seed + 1)), torch, torch.bfloat16)
    bias = to_dev(synth.weights((N,), seed + 2), torch) if epilogue else None
    res = to_dev(orc.bf16_round(synth.activations((M, N), seed + 3)), torch, torch.bfloat16) if epilogue else None
    return X, W, bias, res


def test_static_scratch_gemm_matches_the_scratch_argument_form():
    torch, zo = gpu()
    cases = [(384, 1024, 4096, 4, True), (200, 516, 2048, 2, False), (384, 1024, 2752, 1, True)]
    for i, (M, N, K, ranges, epilogue) in enumerate(cases):
        assert zo.zo_gemm_nt_splitk_ranges(M, N, K) == ranges
        assert zo.zo_gemm_nt_splitk_scratch_bytes(M, N, K) <= zo.zo_gemm_nt_splitk_static_max_bytes()
        X, W, bias, res = _case(torch, zo, M, N, K, 1200 + 10 * i, epilogue)
        want = zo.zo_gemm_nt_fused_splitk(X, W, bias, res, relu=epilogue)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)      # count of allocation requests so far
        got = zo.zo_gemm_nt_fused_splitk_static(X, W, Y, bias, res, relu=epilogue)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before
        assert torch.equal(got, want), (M, N, K)                       # same kernels, same ranges: the same bits
        ref = X.float().cpu().numpy().astype(np.float64) @ W.float().cpu().numpy().astype(np.float64).T
        if epilogue:
            ref = np.maximum(ref + bias.cpu().numpy(), 0.0) + res.float().cpu().numpy()
        err = np.abs(got.float().cpu().numpy() - ref)
        assert np.all(err <= 2.0 ** -8 * np.abs(ref) + 1e-5 * np.sqrt(K) + 1e-6)


def test_static_scratch_gemm_rejects_what_the_array_cannot_hold():
    torch, zo = gpu()
    M, N, K = 1280, 2048, 16384                # 4 ranges x 1280 x 2048 x 4 B = 40 MiB of partial sums
    assert zo.zo_gemm_nt_splitk_scratch_bytes(M, N, K) > zo.zo_gemm_nt_splitk_static_max_bytes()
    X = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((N, K), dtype=torch.bfloat16, device="cuda")
    Y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(zo.ZoError) as e:
        zo.zo_gemm_nt_fused_splitk_static(X, W, Y)
    assert e.value.status == 6                 # ZO_EWORKSPACE
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())              # nothing was launched
