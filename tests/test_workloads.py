"""The seeded input generators: shapes, zero ratios and structure as the recipe states (CPU only)."""
import numpy as np
import pytest

import workloads


def test_layer_inputs_are_deterministic_and_have_the_stated_zero_ratio():
    layer, x, w = workloads.make_layer_inputs(1, 1, 1)
    layer2, x2, w2 = workloads.make_layer_inputs(1, 1, 1)
    assert np.array_equal(x, x2) and np.array_equal(w, w2)
    assert x.dtype == np.float32 and w.dtype == np.float32
    assert x.shape == (1, layer.C, layer.H, layer.W) and w.shape == (layer.K, layer.Cg, layer.R, layer.S)
    assert abs(float((x == 0).mean()) - layer.zero_ratio) < 0.01
    assert (x >= 0).all()


def test_per_channel_ratios_stay_in_their_range():
    layer, x, _ = workloads.make_layer_inputs(2, 1, 2)
    lo, hi = layer.per_channel
    zc = (x == 0).mean(axis=(0, 2, 3))
    assert (zc > lo - 0.03).all() and (zc < hi + 0.03).all()


@pytest.mark.parametrize("z", [0.3, 0.7, 0.9])
def test_clustered_structure_keeps_the_overall_ratio_and_adds_dead_planes_and_patches(z):
    base = workloads.CONFIGS[4]["layers"][0].with_zero_ratio(z)
    _, xi, _ = workloads.make_layer_inputs(4, 0, 4, base)
    _, xc, _ = workloads.make_layer_inputs(4, 0, 4, base.with_structure("clustered"))
    zi, zc = xi == 0, xc == 0
    assert abs(float(zc.mean()) - z) < 0.02 and abs(float(zi.mean()) - z) < 0.02
    dead = zc.all(axis=(2, 3)).mean()
    assert abs(float(dead) - 0.3 * z) < 0.05
    # all-zero runs of four neighbours are far more common than with independent zeros
    def runs(m):
        return m[:, :, :, :12].reshape(m.shape[0], m.shape[1], m.shape[2], 3, 4).all(axis=4).mean()
    assert runs(zc) > runs(zi) + 0.05


def test_integer_cases_are_integers():
    _, x, w = workloads.make_random_case(5, 2, 8, 6, 6, 4, 3, 3, 1, 1, 1, None, 0.5, True)
    assert np.array_equal(x, np.round(x)) and np.array_equal(w, np.round(w))
    assert x.max() <= 3 and np.abs(w).max() <= 2


def test_single_layer_config_and_chain_are_consistent():
    """Shapes of the stand-ins for the paper's single layers are valid, and in the chain every layer's
    output is the next layer's input."""
    for layer in workloads.CONFIGS[5]["layers"]:
        assert layer.C % layer.groups == 0 and layer.K % layer.groups == 0
        assert layer.OH >= 1 and layer.OW >= 1 and 0.8 <= layer.zero_ratio <= 0.95
    h, c = workloads.CHAIN[0].H, workloads.CHAIN[0].C
    for layer in workloads.CHAIN:
        assert (layer.C, layer.H, layer.W) == (c, h, h)
        c, h = layer.K, layer.OH
        if layer.pool:
            h = (h - layer.pool[0]) // layer.pool[2] + 1
    x, ws = workloads.make_chain_inputs(1, workloads.CHAIN[:2])
    x2, ws2 = workloads.make_chain_inputs(1, workloads.CHAIN[:2])
    assert np.array_equal(x, x2) and all(np.array_equal(a, b) for a, b in zip(ws, ws2))
    assert ws[0].mean() < 0                      # the stated negative shift of the filter mean


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
