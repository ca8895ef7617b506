"""rocket_make_kernels against the oracle's sampler, bit for bit, on the machine that runs the
GPU tests (the sampler is host code, but its decisions must not depend on the host).  Shapes of
workloads 0, 2 and 4 and the odd cases of the host-side test."""
import pytest

import synth
from kernels_of import sampled

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("i", [0, 2, 4])
def test_workload_kernels_bit_exact(i):
    cfg = synth.CONFIGS[i]
    print("sampler workload", i, flush=True)
    h, kr = sampled(synth.seed_k(i), cfg["K"], cfg["C"], cfg["L"])
    assert len(kr["weights"]) == kr["w_off"][-1]
    h.free()


@pytest.mark.parametrize("seed,K,C,L", [
    (2001, 2000, 1, 1000), (0, 64, 3, 11), (2**64 - 1, 64, 9, 4097), (12345, 200, 40, 333), (7, 300, 2, 3000000),
])
def test_odd_shapes_bit_exact(seed, K, C, L):
    h, _ = sampled(seed, K, C, L)
    h.free()
