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
