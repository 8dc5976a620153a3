"""The synthetic workloads: shape arithmetic of the five configurations and generator determinism."""
import numpy as np

import adacomp_workloads as W


def test_shapes():
    expect = {1: (2, 397_000, 794), 2: (6, 1_174_080, 7_965), 3: (54, 25_502_912, 473_215),
              4: (3, 3_312_128, 6_626), 5: (7, 125_235_200, 250_474)}
    for i, (n_layers, n_params, n_bins) in expect.items():
        wl = W.workload(i)
        assert len(wl.layers) == n_layers and wl.n_params == n_params
        assert sum(-(-l.n_elems // l.L_T) for l in wl.layers) == n_bins
        assert all(l.elem_offset % 4 == 0 for l in wl.layers)
    # ResNet-50: 53 convolutions with L_T 50 and one FC with L_T 500 (Table 2 hyper-parameters)
    r50 = W.workload(3)
    assert sum(l.L_T == 50 for l in r50.layers) == 53 and r50.layers[-1].L_T == 500


def test_generator_is_deterministic_and_thread_independent():
    wl = W.workload(2)
    a = W.gradient(wl, 1, 3, seed=0, threads=1)
    b = W.gradient(wl, 1, 3, seed=0, threads=4)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, W.gradient(wl, 2, 3))
    assert not np.array_equal(a, W.gradient(wl, 1, 4))
    assert not np.array_equal(a, W.gradient(wl, 1, 3, seed=1))


def test_distributions():
    g = W.gradient(W.workload(1), 0, 0)
    assert abs(g.std() - 1e-3) < 2e-5
    wl = W.workload(2)
    g = W.gradient(wl, 0, 0)
    for l, s in zip(wl.layers, W.layer_params(wl)):
        assert 1e-4 <= s <= 1e-2
        assert abs(g[l.elem_offset:l.elem_offset + l.n_elems].std() / s - 1) < 0.1
    wl = W.workload(4)
    g = W.gradient(wl, 0, 0)
    frac = np.mean(np.abs(g) > 0.02)            # base sigma 1e-3: only x100 outliers get this large
    assert 0.006 < frac < 0.01
    wl3 = W.custom("lap", [("a", 200_000, 50)], dist="laplace")
    g = W.gradient(wl3, 0, 0)
    b = W.layer_params(wl3)[0]
    assert np.isfinite(g).all() and abs(np.mean(np.abs(g)) / b - 1) < 0.02   # E|x| = b
