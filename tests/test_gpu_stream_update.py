"""GPU parity: perturbation stream (bit-exact) and the seeded update of Eq. 3 (bit-exact)."""
import numpy as np
import pytest

from oracle import zo_oracle as orc
from paper_2509_00031_amd import synth
from gpu_util import gpu, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,tid,n", [(0, 0, 4099), (0x1234567890ABCDEF, 291, 1025), (7, 3, 1), (7, 3, 0)])
def test_philox_words_bit_exact(seed, tid, n):
    torch, zo = gpu()
    got = zo.zo_debug_philox_u32(seed, tid, n).cpu().numpy().view(np.uint32)
    assert np.array_equal(got, orc.philox_words(seed, tid, n))


@pytest.mark.parametrize("seed,tid,start,n", [(0, 0, 0, 100003), (99, 12, 5, 70001), (1 << 40, 2, (1 << 35) + 3, 4097),
                                              (5, 1, 7, 1), (5, 1, 0, 0)])
def test_normals_bit_exact(seed, tid, start, n):
    torch, zo = gpu()
    got = zo.zo_debug_normal(seed, tid, n, start=start).cpu().numpy()
    want = orc.normal(seed, tid, n, start=start)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("n", [0, 5, 8, 1000003, 1 << 22])
def test_update_bit_exact(n):
    torch, zo = gpu()
    w = synth.weights((n,), 21)
    c = np.float32(3.7e-3)
    g = to_dev(w, torch)
    zo.zo_update_tensor(g, seed=77, tensor_id=9, coeff_host=float(c))
    want = orc.update(w.copy(), 77, 9, c)
    assert np.array_equal(g.cpu().numpy().view(np.uint32), want.view(np.uint32))
    # coefficient read from device memory, second update on top
    cdev = to_dev(np.array([-1.25e-3], np.float32), torch)
    zo.zo_update_tensor(g, seed=78, tensor_id=9, coeff_dev=cdev)
    want = orc.update(want, 78, 9, np.float32(-1.25e-3))
    assert np.array_equal(g.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_update_zero_coefficient_is_identity_and_unaligned_rejected():
    torch, zo = gpu()
    w = synth.weights((4096,), 22)
    g = to_dev(w, torch)
    zo.zo_update_tensor(g, 1, 1, coeff_host=0.0)
    assert np.array_equal(g.cpu().numpy(), w)
    with pytest.raises(zo.ZoError) as e:
        zo.zo_update_tensor(g[1:], 1, 1, coeff_host=0.0)
    assert e.value.status == 3
