"""Same inputs twice give bit-identical losses and masters on every route (no atomics anywhere: partial sums of the
split-K and fused kernels and the loss reductions are added in a fixed order)."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,S,no_fused,lightweight,d_ffn", [(2, 24, 0, 0, 512), (2, 24, 1, 0, 512), (4, 96, 0, 0, 512), (2, 24, 0, 1, 512),
                                                            (1, 100, 0, 1, 512), (1, 200, 0, 0, 2048)])   # the last: GEMMs with K split
def test_step_is_bit_reproducible(B, S, no_fused, lightweight, d_ffn):
    torch, zo = gpu()
    kw = dict(n_layers=2, d_model=256, n_heads=4, d_ffn=d_ffn, vocab=512, max_seq=S, w_bits=4, w_group=64, a_bits=8)
    ocfg = orc.Config(orc.ARCH_LLAMA, act_dtype=1, lightweight=lightweight, **kw)
    cfg = zo.make_config(zo.ARCH_LLAMA, act_dtype=zo.ACT_BF16, no_fused=no_fused, lightweight=lightweight, **kw)
    shapes = orc.param_shapes(ocfg)
    params = synth.model_params(shapes, 121)
    trainable = [n.endswith(".wq") or n.endswith(".wv") for n, _, _ in shapes] if lightweight else None
    ids = to_dev(synth.token_ids(B, S, 512, 122), torch)
    runs = []
    for rep in range(2):
        gp = []
        for i, (w, (_, _, q)) in enumerate(zip(params, shapes)):
            if lightweight and q and not trainable[i]:
                gp.append(zo.zo_pack_weight_int4(to_dev(w, torch), 64))
            else:
                gp.append(to_dev(w, torch))
        ctx = zo.Context(cfg, gp, B, S, trainable=trainable)
        outs = [ctx.zo_step(ids, None, B, S, seed=s, eps=1e-3, lr=1e-3).cpu().numpy().copy() for s in (1, 2, 3)]
        if d_ffn == 2048:
            assert ctx.zo_debug_routes() & zo.ROUTE_GEMM_SPLIT_K
        runs.append((outs, [p.cpu().numpy() for p in gp if not isinstance(p, zo.PackedInt4)]))
        ctx.close()
    for a, b in zip(runs[0][0], runs[1][0]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    for a, b in zip(runs[0][1], runs[1][1]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
