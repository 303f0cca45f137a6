"""Randomised parity: seeded draws of shape, bit width, candidate count, mode and
value distribution, each put through the exhaustive search (both routes when the
call is small), the prefix-sum search and the quantizer and compared with the CPU
oracle, group by group and element by element (the helpers of test_gpu_parity).
Sizes are drawn log-uniformly so that most cases take milliseconds and a few span
several tiles."""
import numpy as np
import pytest

from paper_2002_00104_amd import synth
from test_gpu_parity import _list_case, run_both

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available()
    from paper_2002_00104_amd import pwlq
    return pwlq


def _draw(rng, C, K):
    kind = int(rng.integers(0, 7))
    if kind == 0:
        w = rng.standard_normal((C, K))
    elif kind == 1:
        w = rng.laplace(0, 1, (C, K))
    elif kind == 2:
        w = rng.standard_t(2.0, (C, K))
    elif kind == 3:
        w = rng.uniform(-1, 1, (C, K))
    elif kind == 4:
        w = rng.standard_normal((C, K)) * (rng.random((C, K)) < 0.1)         # mostly zeros
    elif kind == 5:
        w = np.round(rng.standard_normal((C, K)) * 3) / 3                      # many exact ties
    else:
        w = rng.standard_normal((C, K)) * np.exp(rng.normal(0, 3, (C, 1)))     # channels of very different scale
    return (w * np.exp(rng.normal(-3, 2))).astype(np.float32), kind


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_single_tensors(P, seed):
    rng = np.random.default_rng(seed)
    for i in range(120):
        bits = int(rng.integers(2, 9))
        mode = int(rng.integers(0, 2))
        K = int(np.exp(rng.uniform(np.log(8), np.log(40000))))
        C = int(rng.integers(1, 12)) if K > 2000 else int(rng.integers(1, 60))
        n = int(np.exp(rng.uniform(np.log(4), np.log(5000))))
        w, kind = _draw(rng, C, K)
        run_both(P, w, bits, n, mode, f"random seed={seed} case={i} kind={kind}")


@pytest.mark.parametrize("seed", [21, 22])
def test_random_tensor_lists(P, seed):
    rng = np.random.default_rng(seed)
    for i in range(30):
        nt = int(rng.integers(2, 30))
        bits = int(rng.integers(2, 7))
        mode = int(rng.integers(0, 2))
        n = int(np.exp(rng.uniform(np.log(8), np.log(2500))))
        tensors = []
        for _ in range(nt):
            K = int(np.exp(rng.uniform(0, np.log(20000))))
            C = int(rng.integers(1, 6)) if K > 1500 else int(rng.integers(1, 40))
            tensors.append(_draw(rng, C, K)[0])
        _list_case(P, tensors, bits, n, mode, f"random list seed={seed} case={i}", packed=True)
