"""GPU parity: causal softmax attention of the decoder forward against the oracle's fp64 softmax.
fp32 storage: generic kernel, 1e-4.  bf16 storage, head dimension 64 / 128: matrix-core kernel;
the probabilities enter the second product as bf16 operands, so besides the storage rounding of
the output (2^-9 relative) each output carries their rounding noise (about as large)."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev, rel_l2

pytestmark = pytest.mark.gpu


def _ref(qkv, B, S, H, dh):
    d = H * dh
    return orc._attention(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], B, S, H, dh)


@pytest.mark.parametrize("B,S,H,dh", [(2, 40, 4, 32), (1, 130, 2, 64), (1, 64, 1, 16), (2, 33, 1, 128)])
def test_attention_fp32(B, S, H, dh):
    torch, zo = gpu()
    qkv = synth.activations((B * S, 3 * H * dh), 71) * 1.5
    out = zo.zo_attention_causal(to_dev(qkv, torch), B, S, H, dh).cpu().numpy()
    ref = _ref(qkv, B, S, H, dh)
    assert rel_l2(out, ref) < 1e-5
    assert np.abs(out - ref).max() < 1e-4 * np.abs(ref).max()


@pytest.mark.parametrize("B,S,H,dh", [(2, 40, 2, 64), (1, 200, 1, 128), (2, 128, 2, 64), (1, 257, 2, 128),
                                      (1, 1024, 1, 128), (3, 64, 1, 64), (1, 1, 1, 64), (2, 96, 3, 32),
                                      (5, 70, 15, 64), (2, 150, 40, 128)])     # more (batch, head) pairs than one chunk of the work list
@pytest.mark.parametrize("sharp", [0.5, 3.0])
def test_attention_bf16(B, S, H, dh, sharp):
    torch, zo = gpu()
    qkv = orc.bf16_round(synth.activations((B * S, 3 * H * dh), 72) * sharp)
    out = zo.zo_attention_causal(to_dev(qkv, torch, torch.bfloat16), B, S, H, dh).float().cpu().numpy()
    ref = _ref(qkv, B, S, H, dh)
    row = np.linalg.norm(out - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert rel_l2(out, ref) < 4e-3, rel_l2(out, ref)
    assert row.max() < 8e-3, row.max()
    # position 0 attends to itself only: output = v[0] exactly
    d = H * dh
    assert np.array_equal(out[0], qkv[0, 2 * d:])


@pytest.mark.parametrize("rise", [4.0, 40.0, 400.0])
@pytest.mark.parametrize("dh", [64, 128])
def test_attention_bf16_growing_scores(rise, dh):
    """Scores that climb by `rise` (natural-log units) from the first key to the last: the kernel moves the reference
    point of its exponentials only when the maximum has outgrown it by 2^8, so a slow climb keeps a stale reference
    for many tiles and a steep one moves it in every tile; the output must not depend on that."""
    torch, zo = gpu()
    B, S, H = 1, 448, 2
    d = H * dh
    qkv = synth.activations((B * S, 3 * d), 73) * 0.25
    ramp = np.linspace(0.0, 1.0, S, dtype=np.float32)
    for h in range(H):
        qkv[:, h * dh] = 4.0                                            # q: one large component ...
        qkv[:, d + h * dh] = ramp * np.float32(rise * np.sqrt(dh) / 4.0)    # ... meets a key component that grows with the position
    qkv = orc.bf16_round(qkv)
    out = zo.zo_attention_causal(to_dev(qkv, torch, torch.bfloat16), B, S, H, dh).float().cpu().numpy()
    ref = _ref(qkv, B, S, H, dh)
    row = np.linalg.norm(out - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert rel_l2(out, ref) < 4e-3, rel_l2(out, ref)
    assert row.max() < 8e-3, row.max()
