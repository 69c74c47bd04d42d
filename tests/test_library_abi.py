"""CPU-only: the C-ABI library loads and exports every symbol the header declares; host-side
argument checks that need no GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2509_00031_amd", "libzoqat.so")


def _declared():
    text = open(os.path.join(ROOT, "include", "zoqat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zo_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.skip("libzoqat.so not built (run __graft_entry__.build())")
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_entry_points(lib):
    from paper_2509_00031_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_host_side_shape_logic(lib):
    from paper_2509_00031_amd import binding as zo
    cfg = zo.make_config(zo.ARCH_LLAMA, n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000, max_seq=1024,
                         w_bits=4, w_group=64, a_bits=8, act_dtype=zo.ACT_BF16)
    assert zo.zo_num_params(cfg) == 1 + 32 * 9 + 2
    total = sum(zo.zo_param_numel(cfg, i) for i in range(zo.zo_num_params(cfg)))
    assert total == 6738415616                         # Llama-2-7B parameter count
    assert zo.zo_param_numel(cfg, 9999) == -1
    ws = zo.zo_workspace_bytes(cfg, 8, 1024)
    assert 2 * 1024 ** 3 < ws < 12 * 1024 ** 3
    opt = zo.make_config(zo.ARCH_OPT, n_layers=24, d_model=2048, n_heads=32, d_ffn=8192, vocab=50272, max_seq=2048,
                         w_bits=4, w_group=128, a_bits=8)
    assert zo.zo_num_params(opt) == 2 + 24 * 16 + 3
    bad = zo.make_config(zo.ARCH_LLAMA, n_layers=1, d_model=100, n_heads=4, d_ffn=256, vocab=64, max_seq=16)
    assert zo.zo_workspace_bytes(bad, 1, 16) == 0      # d_model not a multiple of 8
    assert zo.zo_num_params(zo.make_config(7)) == 0


def test_linear_decay_is_the_oracles(lib):
    """Host function of the library against the oracle's schedule (Appendix, hyperparameter table)."""
    import numpy as np
    from oracle import zo_oracle as orc
    from paper_2509_00031_amd import binding as zo
    for lr0, T in ((5e-7, 10000), (1e-8, 10000), (1e-2, 7)):
        for t in (0, 1, T // 3, T // 2, T - 1):
            assert np.float32(zo.zo_lr_linear_decay(lr0, t, T)) == orc.lr_linear_decay(lr0, t, T)
