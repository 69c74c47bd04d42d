"""GPU parity: the contraction of the quantized linears and one fake-quantized linear layer.
Tolerances: relative l2 error 1e-4 with fp32 storage, 1e-2 with bf16 storage."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev, rel_l2

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,N,K", [(8, 256, 256), (300, 200, 328), (1, 1, 8), (257, 513, 1024), (1024, 768, 512)])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_gemm_nt(M, N, K, dtype):
    torch, zo = gpu()
    X = synth.activations((M, K), 51)
    W = synth.weights((N, K), 52, scale=1.0)
    if dtype == "bf16":
        X, W = orc.bf16_round(X), orc.bf16_round(W)
        td = torch.bfloat16
    else:
        td = torch.float32
    Y = zo.zo_gemm_nt(to_dev(X, torch, td), to_dev(W, torch, td)).float().cpu().numpy()
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    # element-wise: fp32 accumulation over K terms, then storage rounding
    tol = (2.0 ** -8 if dtype == "bf16" else 2.0 ** -20) * np.abs(ref) + 1e-5 * np.sqrt(K)
    assert np.all(np.abs(Y - ref) <= tol)
    assert rel_l2(Y, ref) < (4e-3 if dtype == "bf16" else 1e-6)


def test_gemm_large_tile_path():
    torch, zo = gpu()
    M, N, K = 3000, 2900, 256                      # takes the 256 x 256 tile kernel, ragged in M and N
    X = orc.bf16_round(synth.activations((M, K), 53))
    W = orc.bf16_round(synth.weights((N, K), 54, scale=1.0))
    Y = zo.zo_gemm_nt(to_dev(X, torch, torch.bfloat16), to_dev(W, torch, torch.bfloat16)).float().cpu().numpy()
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.all(np.abs(Y - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4)


@pytest.mark.parametrize("M,N,K", [(3000, 2904, 256), (2051, 4096, 512), (200, 136, 64), (4096, 2048, 128), (3300, 3304, 256),
                                   (3201, 3500, 192)])
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("bias,relu,residual", [(True, False, False), (False, False, True), (True, True, True)])
def test_gemm_fused_epilogue(M, N, K, dtype, bias, relu, residual):
    """Bias / ReLU / in-place residual epilogue, on shapes that take the register-staged kernel (K = 64), the 128 x 128
    and the 256 x 256 tiles of the load-unit pipeline (13 x 13 and more tiles of 256), with (bf16, N a multiple of 8) and
    without (N = 3500) the row-coalesced store path, ragged in M and N."""
    torch, zo = gpu()
    bf = dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    X = synth.activations((M, K), 55)
    W = synth.weights((N, K), 56, scale=1.0)
    R = synth.activations((M, N), 57)
    b = synth.weights((N,), 58, scale=1.0)
    if bf:
        X, W, R = orc.bf16_round(X), orc.bf16_round(W), orc.bf16_round(R)
    Y = to_dev(R, torch, td) if residual else None           # residual stream updated in place
    out = zo.zo_gemm_nt_fused(to_dev(X, torch, td), to_dev(W, torch, td), to_dev(b, torch) if bias else None,
                              Y, relu, Y).float().cpu().numpy()
    acc = X.astype(np.float64) @ W.astype(np.float64).T
    mag = np.abs(acc)
    if bias:
        acc = acc + b.astype(np.float64)
    if relu:
        acc = np.maximum(acc, 0.0)
    if residual:
        acc = acc + R.astype(np.float64)
    tol = (2.0 ** -8 if bf else 2.0 ** -20) * (np.abs(acc) + mag) + 1e-5 * np.sqrt(K)
    assert np.all(np.abs(out - acc) <= tol)


@pytest.mark.parametrize("M,N,K,ranges", [(384, 1024, 4096, 4), (200, 516, 2048, 2), (130, 260, 8192, 8), (384, 1024, 2752, 1),
                                          (300, 1030, 4096, 1), (4096, 4096, 4096, 1)])
@pytest.mark.parametrize("bias,relu,residual", [(False, False, False), (True, True, True)])
def test_gemm_split_k(M, N, K, ranges, bias, relu, residual):
    """The K-split form of the 128 x 128-tile kernel (few tokens, narrow N, long K): 2, 4 and 8 ranges, ragged M and N, and
    shapes the planner leaves whole (K tiles not divisible, N not a multiple of 4, enough tiles), which must then equal the
    unsplit entry point bit for bit.  Against the fp64 product; and against the unsplit kernel, from which only the order of
    the fp32 additions differs."""
    torch, zo = gpu()
    assert zo.zo_gemm_nt_splitk_ranges(M, N, K) == ranges
    td = torch.bfloat16
    X = orc.bf16_round(synth.activations((M, K), 61))
    W = orc.bf16_round(synth.weights((N, K), 62, scale=1.0))
    R = orc.bf16_round(synth.activations((M, N), 63))
    b = synth.weights((N,), 64, scale=1.0)
    Xd, Wd, bd = to_dev(X, torch, td), to_dev(W, torch, td), to_dev(b, torch) if bias else None
    Y = to_dev(R, torch, td) if residual else None
    got = zo.zo_gemm_nt_fused_splitk(Xd, Wd, bd, Y, relu, Y).float().cpu().numpy()
    Y2 = to_dev(R, torch, td) if residual else None
    whole = zo.zo_gemm_nt_fused(Xd, Wd, bd, Y2, relu, Y2).float().cpu().numpy()
    acc = X.astype(np.float64) @ W.astype(np.float64).T
    mag = np.abs(acc)
    if bias:
        acc = acc + b.astype(np.float64)
    if relu:
        acc = np.maximum(acc, 0.0)
    if residual:
        acc = acc + R.astype(np.float64)
    tol = 2.0 ** -8 * (np.abs(acc) + mag) + 1e-5 * np.sqrt(K)
    assert np.all(np.abs(got - acc) <= tol)
    if ranges == 1:
        assert np.array_equal(got, whole)
    else:
        # same sums in another order: the fp32 sums differ by their accumulated rounding (a few 2^-24 of the largest running
        # sum per addition), the outputs by at most one bf16 step more, and only where a sum straddles a rounding boundary
        assert np.all(np.abs(got - whole) <= 2.0 ** -7 * np.abs(whole) + 1e-4 * (mag + np.abs(acc)) + 1e-4)
        assert np.mean(got != whole) < 0.05


@pytest.mark.parametrize("dtype,tol", [("fp32", 1e-4), ("bf16", 1e-2)])
@pytest.mark.parametrize("M,N,K,wb,g,ab", [(8, 256, 256, 4, 64, 8), (100, 72, 512, 2, 64, 16), (33, 130, 384, 4, 128, 4)])
def test_linear_fakequant(dtype, tol, M, N, K, wb, g, ab):
    torch, zo = gpu()
    X = synth.activations((M, K), 55)
    W = synth.weights((N, K), 56)
    bias = synth.weights((N,), 57)
    bf = dtype == "bf16"
    if bf:
        X = orc.bf16_round(X)
    xd = to_dev(X, torch, torch.bfloat16 if bf else torch.float32)
    for eps in (1e-3, -1e-3):
        Y = zo.zo_linear_fakequant(xd, to_dev(W, torch), to_dev(bias, torch), wb, g, ab, 0, seed=11, tensor_id=4,
                                   eps_signed=eps).float().cpu().numpy()
        what = orc.fakequant_weight(W, wb, g, 11, 4, np.float32(eps), round_bf16=bf, want_codes=False)["what"]
        xhat = orc.fakequant_act(X, ab, False, round_bf16=bf, want_codes=False)["xhat"]
        ref = orc.linear(xhat, what, bias)
        assert rel_l2(Y, ref) < tol
        assert np.abs(Y - ref).max() <= (2.0 ** -7 if bf else 1e-5) * np.abs(ref).max()
