"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI binding, run the
oracle on the same host arrays, compare to the stated bars."""
import numpy as np
import torch

import oracle
import paper_1909_09927_amd as sconv

# fp32 outputs must lie within TOL * sum|x*w| of the fp64 result (per output element).
TOL = 1e-4


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_forward(layer, x, w, relu=True, integer_exact=False):
    y = sconv.sconv_forward(to_dev(x), to_dev(w), layer.stride, layer.pad, layer.groups, relu=relu)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    ref, scale = oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=relu)
    assert got.shape == ref.shape
    err = np.abs(got - ref)
    if integer_exact:
        assert np.array_equal(got, ref), f"max err {err.max()} on integer-valued inputs"
    bad = err > TOL * scale
    assert not bad.any(), (f"{layer.name}: {bad.sum()} of {bad.size} outputs beyond {TOL}*sum|xw|; "
                           f"worst ratio {np.max(err / np.maximum(scale, 1e-300)):.3e}")
    return float(np.max(err / np.maximum(scale, 1e-30)))


def check_pool_forward(layer, x, w, integer_exact=False):
    y = sconv.sconv_pool_forward(to_dev(x), to_dev(w), layer.pool, layer.stride, layer.pad, layer.groups)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    ref, scale = oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
    assert got.shape == ref.shape
    err = np.abs(got - ref)
    if integer_exact:
        assert np.array_equal(got, ref), f"max err {err.max()} on integer-valued inputs"
    bad = err > TOL * scale
    assert not bad.any(), (f"{layer.name}: {bad.sum()} of {bad.size} pooled outputs beyond tolerance; "
                           f"worst ratio {np.max(err / np.maximum(scale, 1e-300)):.3e}")
    return float(np.max(err / np.maximum(scale, 1e-30)))


def check_encode(layer, x, w_shape, fmt):
    pool = layer.pool if fmt == sconv.FMT_PECR else None
    v, i, c = sconv.sconv_encode(to_dev(x), w_shape, fmt, layer.stride, layer.pad, layer.groups, pool)
    torch.cuda.synchronize()
    rv, ri, rc = oracle.encode(x, w_shape, fmt, layer.stride, layer.pad, layer.groups, pool)
    gv, gi, gc = v.cpu().numpy(), i.cpu().numpy(), c.cpu().numpy()
    assert gc.shape == rc.shape and gv.shape == rv.shape
    assert np.array_equal(gc, rc), "count differs"
    assert np.array_equal(gi, ri), "index differs"
    # bit-exact values, sign of zero included
    assert np.array_equal(gv.view(np.uint32), rv.view(np.uint32)), "values differ"
