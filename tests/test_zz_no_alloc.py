"""The entry point that allocates nothing, sconv_forward_static, against sconv_forward on the same
inputs: same split through scratch (here the library's static array instead of a lent workspace), so
the results must agree to the conv tolerance (1e-4 * sum|x*w| per element, the bar every fp32 output is
held to) - and bit for bit when both take the same plan, which the pinned decomposition makes sure of.
Two calls in a row, the second on a smaller problem: the array keeps the first call's partial sums and
nothing may leak from them."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1909_09927_amd as sconv
import workloads
from parity import TOL, to_dev

pytestmark = pytest.mark.gpu


def _mk(seed, shp, z=0.7):
    N, C, H, W, K, R, S, stride, pad, groups, pool = shp
    return workloads.make_random_case(seed, N, C, H, W, K, R, S, stride, pad, groups, pool, z, False)

# (shape, pinned tap decomposition "wavefronts,slices,workgroups per tile"): deep batch-1 layers, split
CASES = [
    ((2, 512, 7, 7, 512, 3, 3, 1, 1, 1, None), "8,8,4"),
    ((1, 256, 7, 7, 128, 3, 3, 1, 1, 1, None), "8,8,2"),
]


def test_static_scratch_entry_point_matches_the_lent_workspace_path(device, monkeypatch):
    monkeypatch.setenv("SCONV_VARIANT", "tap")
    L = sconv.lib()
    for i, (shp, split) in enumerate(CASES):
        monkeypatch.setenv("SCONV_TAP_SPLIT", split)
        layer, x, w = _mk(7100 + i, shp)
        xd, wd = to_dev(x), to_dev(w)
        ref_call = sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True)   # lent workspace
        out = torch.full_like(ref_call, float("nan"))
        desc = sconv.desc_for(xd, wd, layer.stride, layer.pad, layer.groups, None, True)
        rc = L.sconv_forward_static(ctypes.byref(desc), xd.data_ptr(), wd.data_ptr(), out.data_ptr(),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == sconv.SCONV_OK, sconv.strerror(rc)
        torch.cuda.synchronize()
        ref, scale = oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
        got = out.cpu().numpy().astype(np.float64)
        assert (np.abs(got - ref_call.cpu().numpy()) <= TOL * scale).all()
        assert (np.abs(got - ref) <= TOL * scale).all()
        assert torch.equal(out, ref_call), "same plan, same order of additions"


def test_static_scratch_entry_point_without_pins_and_its_size_limit(device):
    """Default dispatch (whatever plan it takes) on a small layer, then a problem beyond the limit."""
    shp = (1, 512, 7, 7, 256, 3, 3, 1, 1, 1, None)
    layer, x, w = _mk(7200, shp)
    xd, wd = to_dev(x), to_dev(w)
    y = sconv.sconv_forward_static(xd, wd, 1, 1, 1, relu=True)
    torch.cuda.synchronize()
    ref, scale = oracle.conv(x, w, 1, 1, 1, relu=True)
    assert (np.abs(y.cpu().numpy().astype(np.float64) - ref) <= TOL * scale).all()
    big = sconv.make_desc(8, 64, 56, 56, 128, 3, 3, 1, 1, 1, None, True)   # 2 slices = 25.7 MB > 16 MiB
    p = ctypes.c_void_p(xd.data_ptr())
    assert sconv.lib().sconv_forward_static(ctypes.byref(big), p, p, p, None) == sconv.SCONV_ETOOLARGE
    assert "static scratch" in sconv.strerror(sconv.SCONV_ETOOLARGE)
