"""The synthetic workloads take the shapes and sizes the benchmark names."""
import numpy as np

from paper_2002_00104_amd import synth


def test_workload_sizes():
    want = {1: (1, 64, 36864), 2: (54, 27560, 25502912), 3: (53, 18056, 3469760),
            4: (95, 95, 23799136), 5: (6, 38400, 157286400)}
    for i, (nt, ng, ne) in want.items():
        wl = synth.workload(i)
        assert (wl.n_tensors, wl.n_groups, wl.n_elements) == (nt, ng, ne)
    k9 = sum(c for c, k in map(synth.as_ck, synth.workload(3).shapes) if k == 9)
    assert k9 == 7136


def test_tensors_are_seeded_and_fp32():
    wl = synth.workload(2)
    a, b = wl.tensor(3), wl.tensor(3)
    assert a.dtype == np.float32 and a.shape == wl.ck(3)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(wl.tensor(4)[:4, :4], a[:4, :4])
    w1 = synth.workload(1).tensor(0)
    assert w1.shape == (64, 576) and abs(np.abs(w1).mean() - 0.05) < 0.002
    w5 = synth.workload(5).tensor(0)[:64]
    assert 1e-4 < (np.abs(w5) > 0.3).mean() < 5e-4        # the x10 outliers
