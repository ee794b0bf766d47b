"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on
the same seeded inputs.  Encoding arrays bit-exact; conv / pooled outputs within 1e-4*sum|x*w|;
integer-valued inputs bit-exact."""
import numpy as np
import pytest
import torch

import workloads
import paper_1909_09927_amd as sconv
from parity import check_encode, check_forward, check_pool_forward, to_dev

pytestmark = pytest.mark.gpu

# (N, C, H, W, K, R, S, stride, pad, groups, pool)
SMALL = [
    (1, 1, 5, 5, 1, 3, 3, 1, 0, 1, (2, 2, 1)),          # the paper's figure geometry
    (2, 3, 7, 6, 4, 3, 3, 1, 1, 1, (2, 2, 2)),
    (1, 4, 9, 8, 6, 3, 2, 2, 1, 2, (2, 2, 1)),          # non-square kernel, stride 2, groups
    (2, 6, 8, 8, 9, 1, 1, 1, 0, 3, (3, 3, 2)),          # 1x1 grouped, 3x3 pooling (9 windows)
    (1, 2, 10, 11, 3, 5, 3, 3, 2, 1, (2, 1, 1)),        # stride 3, pad 2
    (1, 8, 6, 6, 8, 3, 3, 1, 1, 8, (2, 2, 2)),          # depthwise
    (3, 5, 4, 9, 2, 2, 4, 2, 1, 1, (1, 2, 1)),
    (2, 40, 19, 23, 70, 3, 3, 1, 1, 1, (2, 2, 2)),      # several tiles, ragged tails in K and windows
    (1, 33, 17, 13, 130, 3, 3, 1, 1, 1, (3, 2, 2)),
    (1, 64, 30, 30, 300, 1, 1, 1, 0, 1, (2, 2, 2)),     # K beyond one 256-filter tile
    (2, 96, 14, 14, 96, 3, 3, 1, 1, 3, (2, 2, 2)),
    (1, 16, 21, 21, 20, 7, 7, 2, 3, 1, (2, 2, 2)),      # large kernel
    (1, 8, 40, 40, 16, 3, 3, 1, 1, 1, (7, 7, 3)),       # 49-result pooling window
    # 3x3 / stride 1 / pad 1 with whole 8- or 16-channel chunks: the element-stationary kernel
    (2, 32, 19, 23, 70, 3, 3, 1, 1, 1, (2, 2, 2)),      # one filter per lane, ragged filter block
    (1, 16, 28, 28, 32, 3, 3, 1, 1, 1, (2, 2, 2)),      # half-empty filter block
    (2, 24, 17, 30, 200, 3, 3, 1, 1, 1, (2, 2, 2)),     # two filters per lane, ragged block, odd sizes
    (3, 64, 7, 7, 128, 3, 3, 1, 1, 1, (2, 2, 2)),       # whole-map 7x7 tile
    (2, 48, 14, 14, 192, 3, 3, 1, 1, 1, (2, 2, 2)),     # 14-wide pooled tile
    (2, 64, 14, 14, 64, 3, 3, 1, 1, 2, (2, 2, 2)),      # grouped
    (1, 256, 9, 12, 256, 3, 3, 1, 1, 1, (2, 2, 2)),     # many chunks, channel slices
    (9, 16, 6, 5, 130, 3, 3, 1, 1, 1, (2, 2, 2)),       # maps smaller than a tile
    # 1x1 / stride 1 / pad 0 with whole 64-channel chunks: the pointwise matrix-core kernel
    (2, 64, 9, 11, 70, 1, 1, 1, 0, 1, (2, 2, 2)),       # ragged filter block, odd plane size
    (1, 128, 28, 28, 128, 1, 1, 1, 0, 1, (2, 2, 2)),
    (3, 256, 7, 7, 64, 1, 1, 1, 0, 2, (2, 2, 2)),       # grouped, plane smaller than a tile
    (1, 192, 30, 58, 40, 1, 1, 1, 0, 1, (2, 2, 2)),     # pooled tiles: ragged columns (58 = 2*28 + 2)
    (2, 64, 5, 8, 64, 1, 1, 1, 0, 1, (2, 2, 2)),        # odd height: last row unpooled
    # 3x3 / stride 2 / pad 1: the stride-2 tiles of the same kernel
    (2, 32, 19, 23, 70, 3, 3, 2, 1, 1, (2, 2, 2)),      # odd sizes, one filter per lane
    (1, 48, 28, 28, 160, 3, 3, 2, 1, 1, (2, 2, 2)),     # two filters per lane, ragged block
    (3, 64, 8, 9, 64, 3, 3, 2, 1, 4, (2, 2, 1)),        # grouped, tiny maps
]


def _untuned(plan_name):
    """"variant/model" or "variant/model:what the cost model would launch"; a tuned one ends in a
    decomposition or in "/kept"."""
    parts = plan_name.split("/")
    return len(parts) >= 2 and parts[1].startswith("model") and parts[-1] != "kept"


def _mk(seed, shp, z=0.7, integer=False):
    N, C, H, W, K, R, S, stride, pad, groups, pool = shp
    return workloads.make_random_case(seed, N, C, H, W, K, R, S, stride, pad, groups, pool, z, integer)


@pytest.mark.parametrize("shp", SMALL)
def test_encode_ecr_bit_exact(device, shp):
    layer, x, w = _mk(101, shp)
    check_encode(layer, x, w.shape, sconv.FMT_ECR)


ENCODE_LARGE = [
    (1, 5, 60, 61, 4, 3, 3, 1, 1, 1, (2, 2, 2)),        # a map above the tiled kernel's threshold, ragged last tile
    (2, 8, 50, 47, 4, 5, 3, 2, 2, 2, (3, 3, 2)),        # stride 2, grouped, overlapping 3x3 pooling windows
    (1, 400, 15, 15, 8, 1, 1, 1, 0, 1, (2, 2, 1)),      # long 1x1 channel loop: several staged chunks
    (1, 3, 70, 9, 2, 7, 7, 3, 3, 1, (2, 1, 1)),         # tall narrow map, large kernel, stride 3
]


@pytest.mark.parametrize("which", ["tile", "rows"])
@pytest.mark.parametrize("shp", SMALL + ENCODE_LARGE)
def test_encode_both_kernels_bit_exact(device, monkeypatch, shp, which):
    """The tiled conversion kernel (input box staged in LDS) and the window-per-wavefront one, each
    forced on every shape (a box too large for the staging buffer falls back to the latter)."""
    monkeypatch.setenv("SCONV_ENCODE", which)
    layer, x, w = _mk(120, shp)
    check_encode(layer, x, w.shape, sconv.FMT_ECR)
    check_encode(layer, x, w.shape, sconv.FMT_PECR)
    layer, x, w = _mk(121, shp, z=0.0)
    check_encode(layer, x, w.shape, sconv.FMT_ECR)
    layer, x, w = _mk(122, shp, z=1.0)
    check_encode(layer, x, w.shape, sconv.FMT_PECR)


@pytest.mark.parametrize("shp", ENCODE_LARGE)
def test_encode_large_maps_bit_exact(device, shp):
    layer, x, w = _mk(123, shp)
    check_encode(layer, x, w.shape, sconv.FMT_ECR)
    check_encode(layer, x, w.shape, sconv.FMT_PECR)


@pytest.mark.parametrize("shp", SMALL)
def test_encode_pecr_bit_exact(device, shp):
    layer, x, w = _mk(102, shp)
    check_encode(layer, x, w.shape, sconv.FMT_PECR)


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shp", SMALL)
def test_forward_parity(device, shp, relu):
    layer, x, w = _mk(103, shp)
    check_forward(layer, x, w, relu=relu)


@pytest.mark.parametrize("shp", SMALL)
def test_pool_forward_parity(device, shp):
    layer, x, w = _mk(104, shp)
    check_pool_forward(layer, x, w)


@pytest.mark.parametrize("shp", SMALL)
def test_integer_inputs_bit_exact(device, shp):
    layer, x, w = _mk(105, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    check_pool_forward(layer, x, w, integer_exact=True)


@pytest.mark.parametrize("z", [0.0, 0.5, 0.95, 1.0])
def test_sparsity_extremes(device, z):
    shp = (2, 24, 15, 15, 40, 3, 3, 1, 1, 1, (2, 2, 2))
    layer, x, w = _mk(106, shp, z=z)
    if z == 1.0:
        assert not x.any()
    check_encode(layer, x, w.shape, sconv.FMT_ECR)
    check_encode(layer, x, w.shape, sconv.FMT_PECR)
    check_forward(layer, x, w, relu=False)
    check_pool_forward(layer, x, w)


def test_negative_zero_denormals_and_negative_values(device):
    shp = (1, 4, 9, 9, 8, 3, 3, 1, 1, 1, (2, 2, 2))
    layer, x, w = _mk(107, shp)
    x = x.copy()
    x[0, 0, 0, :3] = [-0.0, 1e-42, -2.5]
    x[0, 1, 4, 4] = -0.0
    check_encode(layer, x, w.shape, sconv.FMT_ECR)
    check_forward(layer, x, w, relu=False)


def test_tiny_config(device):
    layer, x, w = workloads.make_layer_inputs(0, 0, 1)
    check_encode(layer, x, w.shape, sconv.FMT_ECR)
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)


def _layers(ci):
    return list(enumerate(workloads.CONFIGS[ci]["layers"]))


@pytest.mark.parametrize("ci,li", [(ci, li) for ci in (1, 2, 3, 4, 5) for li, _ in _layers(ci)])
def test_benchmark_layers_batch1(device, ci, li):
    """Every layer shape of the benchmark configs at batch 1, whole tensor against the oracle."""
    layer, x, w = workloads.make_layer_inputs(ci, li, 1)
    if layer.pool:
        check_pool_forward(layer, x, w)
    else:
        check_forward(layer, x, w, relu=True)


def _full_size_cases():
    out = []
    for ci in (1, 2, 3, 4, 5):
        N = max(workloads.CONFIGS[ci]["batches"])
        for li, _ in _layers(ci):
            out.append((ci, li, N))
    return out


def _run_layer(layer, xd, wd, **kw):
    if layer.pool:
        return sconv.sconv_pool_forward(xd, wd, layer.pool, layer.stride, layer.pad, layer.groups, **kw)
    return sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True, **kw)


def _whole_tensor_check(layer, x, w, got):
    """Every output of a layer against the oracle (fp64, all host cores): the bar of every fp32 result."""
    import oracle
    if layer.pool:
        ref, scale = oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
    else:
        ref, scale = oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
    assert got.shape == ref.shape
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > 1e-4 * scale
    assert not bad.any(), f"{layer.name}: {int(bad.sum())} of {bad.size} outputs beyond 1e-4*sum|xw|, first at {np.argwhere(bad)[0]}"


@pytest.mark.parametrize("ci,li,N", _full_size_cases())
def test_benchmark_layers_full_batch_whole_tensor(device, ci, li, N):
    """Every benchmark layer at its largest batch with the plan the static rules give it (what
    `bench.py --no-tune` times): the WHOLE output tensor against the oracle (0.3-1.5 s of the host's cores
    per layer), plus properties of the whole tensor (ReLU range, an all-zero image gives zero, same result
    when called twice)."""
    layer, x, w = workloads.make_layer_inputs(ci, li, N)
    x[N - 1] = 0                                   # one all-zero image: its outputs must be exactly 0
    xd, wd = to_dev(x), to_dev(w)
    y = _run_layer(layer, xd, wd)
    y2 = _run_layer(layer, xd, wd)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    got = y.cpu().numpy()
    assert (got >= 0).all() and np.isfinite(got).all()
    assert not got[N - 1].any()
    _whole_tensor_check(layer, x, w, got)


_FLUSH = None


@pytest.mark.parametrize("ci,li,N", _full_size_cases())
def test_benchmark_layers_full_batch_tuned_plan(device, ci, li, N):
    """The launch configuration the default `bench.py` run times: workspace lent, caches evicted through a
    flush buffer while sconv_tune ranks every variant and decomposition, then the remembered plan - whatever
    it is - on bench.py's own sampled comparison with the oracle and on the whole tensor."""
    import bench
    global _FLUSH
    if _FLUSH is None:
        _FLUSH = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    layer, x, w = workloads.make_layer_inputs(ci, li, N)
    xd, wd = to_dev(x), to_dev(w)
    try:
        ms, plan = sconv.sconv_tune(xd, wd, layer.stride, layer.pad, layer.groups, layer.pool, relu=True, flush=_FLUSH)
        assert ms > 0 and plan
        y = _run_layer(layer, xd, wd)
        y2 = _run_layer(layer, xd, wd)
        torch.cuda.synchronize()
    finally:
        sconv.sconv_tune_reset()
    assert torch.equal(y, y2), plan
    got = y.cpu().numpy()
    assert (got >= 0).all() and np.isfinite(got).all()
    r = bench.sampled_check(layer, x, w, got, 2000 * ci + li)     # what bench.py itself checks before timing
    assert r["checked"] >= 4000 and r["failed"] == 0, (plan, r)
    _whole_tensor_check(layer, x, w, got)


# Pooled 3x3 layers with several staged chunks per channel loop and several channel slices: the one-kernel
# fused tiles (no workspace: nothing can be split), the same with a workspace, and every pooled geometry
# of both element-stationary kernels pinned.
POOLED_DEEP = [
    (2, 256, 14, 14, 128, 3, 3, 1, 1, 1, (2, 2, 2)),     # 16 chunks of 16 channels, two filter blocks
    (1, 96, 12, 20, 64, 3, 3, 1, 1, 1, (2, 2, 2)),       # 4x6 tiles with halo, ragged tile columns
    (3, 64, 14, 14, 200, 3, 3, 1, 1, 2, (2, 2, 2)),      # grouped, ragged filter block
]


@pytest.mark.parametrize("ws", ["lent", "none", "own"])
@pytest.mark.parametrize("shp", POOLED_DEEP)
def test_fused_pooling_with_and_without_a_workspace(device, shp, ws):
    import oracle
    layer, x, w = _mk(310, shp)
    xd, wd = to_dev(x), to_dev(w)
    kw = {}
    if ws == "none":
        kw["ws"] = None
    elif ws == "own":
        kw["ws"] = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    y = sconv.sconv_pool_forward(xd, wd, layer.pool, layer.stride, layer.pad, layer.groups, **kw)
    torch.cuda.synchronize()
    ref, scale = oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
    assert (np.abs(y.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


@pytest.mark.parametrize("geom,split", [("p4x14k1", "16,16"), ("p4x14k1", "8,2"), ("p4x14k2", "8,4"), ("p4x6k1", "16,8"),
                                        ("p4x6k2", "8,8"), ("p4x14k1t", "16,16"), ("p4x14k1t", "8,1"),
                                        ("p4x6k1t", "16,4"), ("p4x6k2t", "8,8"), ("p2x14k2t", "16,16"),
                                        ("p2x14k2t", "8,2"), ("p2x14k1t", "16,8"), ("p2x14hk1t", "8,8"), ("p2x14hk1t", "16,2"),
                                        ("p2x14hk2t", "8,4")])
@pytest.mark.parametrize("shp", POOLED_DEEP)
def test_pooled_tile_geometries_of_the_element_stationary_kernels(device, monkeypatch, shp, geom, split):
    """One kernel computes convolution, ReLU and pooling (no split: the pinned decomposition has one
    workgroup per tile), with channel loops of several chunks and up to 16 channel slices."""
    import oracle
    if "x14" in geom and shp[3] != 14:
        pytest.skip("tile spans a 14-wide map")
    if "k2" in geom and shp[4] // shp[9] <= 64:
        pytest.skip("two filters per lane need more than 64 filters per group")
    monkeypatch.setenv("SCONV_VARIANT", "tap")
    monkeypatch.setenv("SCONV_TAP_GEOM", geom)
    monkeypatch.setenv("SCONV_TAP_SPLIT", split)
    layer, x, w = _mk(311, shp)
    xd, wd = to_dev(x), to_dev(w)
    y = sconv.sconv_pool_forward(xd, wd, layer.pool, layer.stride, layer.pad, layer.groups)
    torch.cuda.synchronize()
    ref, scale = oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
    assert (np.abs(y.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


BIAS_SHAPES = [SMALL[i] for i in range(0, len(SMALL), 3)] + [
    (1, 512, 7, 7, 512, 3, 3, 1, 1, 1, None),            # split across workgroups: the adding kernel applies it
    (2, 256, 14, 14, 128, 3, 3, 1, 1, 1, (2, 2, 2)),
    (1, 64, 13, 13, 96, 3, 3, 1, 1, 1, (3, 3, 2)),       # overlapping pooling windows (general kernel)
]


@pytest.mark.parametrize("variant", [None, "rows", "gen"])
@pytest.mark.parametrize("shp", BIAS_SHAPES)
def test_bias_is_added_before_the_relu_in_every_kernel(device, monkeypatch, shp, variant):
    """sconv_forward_bias / sconv_pool_forward_bias against the oracle's layer-with-bias definition:
    through the default dispatch (whatever specialised kernel the shape gets), the general vector kernel
    and the general matrix kernel; ReLU on and off; negative biases large enough to flip signs."""
    import oracle
    if variant:
        monkeypatch.setenv("SCONV_VARIANT", variant)
    layer, x, w = _mk(340, shp)
    rng = np.random.default_rng(340)
    b = (rng.standard_normal(shp[4]) * 0.5).astype(np.float32)
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    for relu in (True, False):
        y = sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=relu, bias=bd)
        torch.cuda.synchronize()
        ref, scale = oracle.conv_bias(x, w, b, layer.stride, layer.pad, layer.groups, relu=relu)
        assert (np.abs(y.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()
    if layer.pool:
        z = sconv.sconv_pool_forward(xd, wd, layer.pool, layer.stride, layer.pad, layer.groups, bias=bd)
        torch.cuda.synchronize()
        ref, scale = oracle.conv_pool_bias(x, w, b, layer.pool, layer.stride, layer.pad, layer.groups)
        assert (np.abs(z.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


PAIRS = [
    # (N, C1, H, W, K1, R1, S1, stride1, pad1, pool1, K2, R2, S2, stride2, pad2, pool2)
    (3, 1, 28, 28, 20, 5, 5, 1, 0, (2, 2, 2), 50, 5, 5, 1, 0, (2, 2, 2)),      # LeNet conv1+pool -> conv2+pool
    (2, 3, 13, 11, 40, 3, 3, 1, 1, None, 33, 3, 3, 2, 1, None),                # no pooling, ragged filter blocks
    (2, 8, 12, 12, 16, 3, 3, 1, 1, (3, 3, 2), 24, 1, 1, 1, 0, (2, 2, 1)),      # overlapping pooling, then 1x1
]


@pytest.mark.parametrize("with_bias", [False, True])
@pytest.mark.parametrize("pair", PAIRS)
def test_two_layers_with_the_hand_off_in_lds(device, pair, with_bias):
    """sconv_pair_forward: the first layer (checked through its optional copy) against the oracle on x, the
    second against the oracle on the intermediate map the GPU really produced - each layer held to the
    bar of a layer on its own; and the output is the same bits whether or not the copy is asked for."""
    import oracle
    N, C1, H, W, K1, R1, S1, st1, pd1, pool1, K2, R2, S2, st2, pd2, pool2 = pair
    rng = np.random.default_rng(350)
    x = np.where(rng.random((N, C1, H, W)) < 0.5, np.abs(rng.standard_normal((N, C1, H, W))), 0).astype(np.float32)
    w1 = (rng.standard_normal((K1, C1, R1, S1)) * np.sqrt(2.0 / (C1 * R1 * S1))).astype(np.float32)
    w2 = (rng.standard_normal((K2, K1, R2, S2)) * np.sqrt(2.0 / (K1 * R2 * S2))).astype(np.float32)
    b1 = (rng.standard_normal(K1) * 0.1).astype(np.float32) if with_bias else None
    b2 = (rng.standard_normal(K2) * 0.1).astype(np.float32) if with_bias else None
    first = {"stride": st1, "pad": pd1, "pool": pool1, "relu": True}
    second = {"stride": st2, "pad": pd2, "pool": pool2, "relu": True}
    args = (to_dev(x), to_dev(w1), to_dev(w2), first, second)
    kw = {"bias1": to_dev(b1) if with_bias else None, "bias2": to_dev(b2) if with_bias else None}
    y, mid = sconv.sconv_pair_forward(*args, keep_mid=True, **kw)
    y_only, none = sconv.sconv_pair_forward(*args, keep_mid=False, **kw)
    torch.cuda.synchronize()
    assert none is None and torch.equal(y, y_only)

    def layer(inp, w, b, stride, pad, pool):
        zb = b if b is not None else np.zeros(w.shape[0], np.float32)
        if pool:
            return oracle.conv_pool_bias(inp, w, zb, pool, stride, pad, 1)
        return oracle.conv_bias(inp, w, zb, stride, pad, 1, relu=True)

    mid_h = mid.cpu().numpy()
    ref1, sc1 = layer(x, w1, b1, st1, pd1, pool1)
    assert mid_h.shape == ref1.shape and (np.abs(mid_h.astype(np.float64) - ref1) <= 1e-4 * sc1).all()
    assert (mid_h == 0).any()                 # the ReLU made zeros for the second layer to skip
    ref2, sc2 = layer(mid_h, w2, b2, st2, pd2, pool2)
    got = y.cpu().numpy().astype(np.float64)
    assert got.shape == ref2.shape and (np.abs(got - ref2) <= 1e-4 * sc2).all()


def test_pair_that_does_not_fit_or_does_not_chain_is_refused(device):
    x = torch.zeros((1, 64, 56, 56), dtype=torch.float32, device="cuda")
    w1 = torch.zeros((64, 64, 3, 3), dtype=torch.float32, device="cuda")
    w2 = torch.zeros((64, 64, 3, 3), dtype=torch.float32, device="cuda")
    with pytest.raises(sconv.SconvError) as e:
        sconv.sconv_pair_forward(x, w1, w2, {"pad": 1}, {"pad": 1})
    assert e.value.code == sconv.SCONV_EUNSUPPORTED


def test_density_probe_counts_like_the_scan(device):
    """sconv_density counts x != 0 exactly on maps it reads whole (negative zero is a zero, a denormal is
    not), and within sampling error on larger ones."""
    rng = np.random.default_rng(5)
    x = np.where(rng.random((3, 17, 29, 31)) < 0.37, rng.standard_normal((3, 17, 29, 31)), 0.0).astype(np.float32)
    x[0, 0, 0, :4] = [-0.0, 1e-42, 0.0, -3.0]
    counts = sconv.sconv_density(to_dev(x)).cpu().numpy()
    assert counts[0] == x.size and counts[1] == int((x != 0).sum())
    big = np.where(rng.random((8, 256, 56, 56)) < 0.4, 1.0, 0.0).astype(np.float32)    # 6.4 Mi elements: sampled
    c = sconv.sconv_density(to_dev(big)).cpu().numpy()
    assert 3 << 20 <= c[0] <= 4 << 20
    assert abs(c[1] / c[0] - (big != 0).mean()) < 2e-3


@pytest.mark.parametrize("z_hint", [0.0, 0.5, 0.75, 0.95])
@pytest.mark.parametrize("shp", [(16, 64, 28, 28, 128, 3, 3, 1, 1, 1, None), (32, 128, 14, 14, 128, 3, 3, 1, 1, 1, None),
                                 (16, 64, 28, 28, 128, 3, 3, 1, 1, 1, (2, 2, 2))])
def test_density_hint_moves_the_static_choice_and_keeps_parity(device, shp, z_hint):
    """A zero ratio in the descriptor's flags selects the matrix kernels (dense maps), the vector kernel
    (68-92 % zeros) or quad3x3 (sparser still) for launches that fill the matrix tiles; whatever runs meets
    the oracle's bar."""
    layer, x, w = _mk(330, shp, z=z_hint if z_hint < 1 else 0.95)
    xd, wd = to_dev(x), to_dev(w)
    pooled = layer.pool is not None
    d = sconv.desc_for(xd, wd, layer.stride, layer.pad, layer.groups, layer.pool, True, zero_ratio=z_hint)
    name = sconv.sconv_variant_name(d, pooled)
    if 0.68 <= z_hint < 0.92:
        assert name == "tap3x3"
    elif not pooled:
        assert name in ("quad3x3", "wide3x3")
    import oracle
    if pooled:
        y = sconv.sconv_pool_forward(xd, wd, layer.pool, layer.stride, layer.pad, layer.groups, zero_ratio=z_hint)
        ref, scale = oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
    else:
        y = sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True, zero_ratio=z_hint)
        ref, scale = oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
    torch.cuda.synchronize()
    assert (np.abs(y.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


def test_tuned_plans_are_kept_per_density_class(device):
    """Two layers of one shape with different zero ratios (as in a chain: 512 @14x14 at 41 % and at 88 %
    zeros) are tuned with their ratio in the descriptor and keep separate plans; a call without the hint
    still gets the static rules."""
    shp = (4, 128, 14, 14, 128, 3, 3, 1, 1, 1, None)
    try:
        for z in (0.3, 0.9):
            layer, x, w = _mk(331, shp, z=z)
            xd, wd = to_dev(x), to_dev(w)
            sconv.sconv_tune(xd, wd, 1, 1, 1, None, relu=True, zero_ratio=z)
        d_lo = sconv.make_desc(4, 128, 14, 14, 128, 3, 3, 1, 1, 1, None, True, zero_ratio=0.35)
        d_hi = sconv.make_desc(4, 128, 14, 14, 128, 3, 3, 1, 1, 1, None, True, zero_ratio=0.85)
        d_no = sconv.make_desc(4, 128, 14, 14, 128, 3, 3, 1, 1, 1, None, True)
        assert not _untuned(sconv.sconv_plan_name(d_lo)) and not _untuned(sconv.sconv_plan_name(d_hi))
        assert _untuned(sconv.sconv_plan_name(d_no))
    finally:
        sconv.sconv_tune_reset()


TAPT = [
    (2, 64, 14, 14, 96, 3, 3, 1, 1, 1, None),          # ragged filter block
    (1, 128, 28, 28, 128, 3, 3, 1, 1, 1, None),        # 5x7 tiles, ragged last tile row
    (3, 32, 7, 7, 64, 3, 3, 1, 1, 2, None),            # whole-map tile, grouped
    (2, 48, 19, 23, 70, 3, 3, 2, 1, 1, None),          # stride 2, odd sizes
    (1, 256, 7, 7, 256, 3, 3, 1, 1, 1, None),          # deep and small: split over workgroups
]


@pytest.mark.parametrize("split", ["8,1", "8,8", "16,4", "16,16", "8,2,2", "16,4,4"])
@pytest.mark.parametrize("shp", TAPT)
def test_transposed_filter_kernel(device, monkeypatch, shp, split):
    """The element-stationary kernel that reads a transposed copy of the filters (no LDS staging, no
    barrier in the channel loop): every plain geometry that fits the shape, pinned decompositions with
    and without a split across workgroups, ReLU on and off, integer inputs bit for bit."""
    stride = shp[7]
    geoms = ["s2-3x4k1t", "s2-3x4k2t"] if stride == 2 else ["5x7k1t", "5x7k2t"] + (["7x7k1t", "7x7k2t"] if shp[2] == 7 else [])
    monkeypatch.setenv("SCONV_VARIANT", "tap")
    monkeypatch.setenv("SCONV_TAP_SPLIT", split)
    ran = 0
    for geom in geoms:
        if "k2" in geom and shp[4] // shp[9] <= 64:
            continue
        parts = [int(t) for t in split.split(",")]
        if (shp[1] // shp[9]) % (parts[1] * (parts[2] if len(parts) > 2 else 1)):
            continue
        monkeypatch.setenv("SCONV_TAP_GEOM", geom)
        layer, x, w = _mk(320, shp)
        check_forward(layer, x, w, relu=True)
        check_forward(layer, x, w, relu=False)
        layer, x, w = _mk(321, shp, integer=True)
        check_forward(layer, x, w, relu=True, integer_exact=True)
        ran += 1
    if not ran:
        pytest.skip("no geometry of this kernel fits the shape with this decomposition")


def _prep_reference(w, groups):
    """The prepared layout written out on the host: [group][block of 64 filters, even count][channel * 9 + tap][64]."""
    K, Cg, R, S = w.shape
    Kg = K // groups
    blocks = (Kg + 127) // 128 * 2
    out = np.zeros((groups, blocks, Cg * R * S, 64), dtype=np.float32)
    for g in range(groups):
        for k in range(Kg):
            out[g, k // 64, :, k % 64] = w[g * Kg + k].reshape(-1)
    return out.reshape(-1)


@pytest.mark.parametrize("shp", TAPT[:3] + [(1, 32, 8, 8, 200, 3, 3, 1, 1, 1, None)])
def test_filter_prep_writes_the_documented_layout(device, shp):
    """sconv_filter_prep is a permutation with zero padding: bit for bit the layout the header documents."""
    layer, x, w = _mk(325, shp)
    got = sconv.sconv_filter_prep(to_dev(w), groups=shp[9])
    torch.cuda.synchronize()
    ref = _prep_reference(w, shp[9])
    got = got.cpu().numpy().view(np.float32)
    assert got.size >= ref.size and np.array_equal(got[:ref.size].view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("split", [None, "8,1", "8,8", "16,4", "8,2,2"])
@pytest.mark.parametrize("shp", TAPT[:3] + [TAPT[4], (4, 128, 14, 14, 192, 3, 3, 1, 1, 1, (2, 2, 2)),
                                           (2, 128, 28, 28, 128, 3, 3, 1, 1, 1, (2, 2, 2))])
def test_prepared_filters_through_the_transposed_filter_kernel(device, monkeypatch, shp, split):
    """Calls that bring prepared filters (sconv_forward_prep / sconv_pool_forward_prep): the transposed-filter
    kernel reads the caller's copy - with a workspace (split plans), and without any - and must meet the oracle
    like every other path; bias through the same call; integer inputs bit for bit."""
    import oracle
    pooled = shp[10] is not None
    if split is None:
        monkeypatch.delenv("SCONV_VARIANT", raising=False)
    else:
        parts = [int(t) for t in split.split(",")]
        if (shp[1] // shp[9]) % (parts[1] * (parts[2] if len(parts) > 2 else 1)):
            pytest.skip("the slices do not divide the channels")
        monkeypatch.setenv("SCONV_VARIANT", "tap")
        monkeypatch.setenv("SCONV_TAP_SPLIT", split)
    geoms = [None] if split is None else (
        (["p2x14k1t", "p2x14k2t", "p4x14k1t"] if shp[3] == 14 else ["p2x14hk1t", "p4x6k1t"]) if pooled
        else ["5x7k1t", "5x7k1tn", "5x7k2t"] + (["7x7k1t"] if shp[2] == 7 else []))
    own = torch.empty(48 << 20, dtype=torch.uint8, device="cuda")
    ran = 0
    for geom in geoms:
        if geom and "k2" in geom and shp[4] // shp[9] <= 64:
            continue
        if geom:
            monkeypatch.setenv("SCONV_TAP_GEOM", geom)
        for integer in (False, True):
            layer, x, w = _mk(326 + integer, shp, integer=integer)
            b = (np.arange(shp[4]) % 5 - 2).astype(np.float32)
            xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
            wp = sconv.sconv_filter_prep(wd, groups=shp[9])
            assert wp is not None
            if pooled:
                ref, scale = oracle.conv_pool(x, w, layer.pool, 1, 1, shp[9])
                refb, scaleb = oracle.conv_pool_bias(x, w, b, layer.pool, 1, 1, shp[9])
                call = lambda **kw: sconv.sconv_pool_forward(xd, wd, layer.pool, 1, 1, shp[9], wprep=wp, **kw)
            else:
                ref, scale = oracle.conv(x, w, 1, 1, shp[9], relu=True)
                refb, scaleb = oracle.conv_bias(x, w, b, 1, 1, shp[9], relu=True)
                call = lambda **kw: sconv.sconv_forward(xd, wd, 1, 1, shp[9], relu=True, wprep=wp, **kw)
            outs = []
            for what, kw, r, sc in (("no workspace", {}, ref, scale), ("own workspace", {"ws": own}, ref, scale),
                                    ("bias", {"ws": own, "bias": bd}, refb, scaleb)):
                try:
                    outs.append((call(**kw), r, sc, what))
                except sconv.SconvError as e:
                    # a pinned split across workgroups needs the workspace: without one the pinned plan does
                    # not apply and the pinned variant has nothing else to offer
                    assert e.code == sconv.SCONV_EUNSUPPORTED and split is not None, what
            torch.cuda.synchronize()
            for got, r, sc, what in outs:
                g = got.cpu().numpy().astype(np.float64)
                if integer:
                    assert np.array_equal(g, r), f"{geom} {what}: integer inputs must be exact"
                else:
                    err = np.abs(g - r)
                    assert (err <= 1e-4 * sc).all(), f"{geom} {what}: {int((err > 1e-4 * sc).sum())} beyond the bar"
            ran += len(outs)
    if not ran:
        pytest.skip("no geometry of this kernel fits the shape with this decomposition")


def test_prepared_filters_are_ignored_where_no_kernel_reads_them_and_tuned_separately(device):
    """A 1x1 layer has no prepared layout (size 0, the forward call runs as without); plans tuned for calls
    with prepared filters are kept apart from those without."""
    import oracle
    layer, x, w = _mk(328, (2, 64, 14, 14, 64, 1, 1, 1, 0, 1, None))
    assert sconv.sconv_filter_prep(to_dev(w), pad=0) is None
    shp = (8, 128, 14, 14, 128, 3, 3, 1, 1, 1, None)
    layer, x, w = _mk(329, shp)
    xd, wd = to_dev(x), to_dev(w)
    wp = sconv.sconv_filter_prep(wd)
    own = torch.empty(48 << 20, dtype=torch.uint8, device="cuda")
    try:
        ms, plan = sconv.sconv_tune(xd, wd, 1, 1, 1, None, relu=True, wprep=wp, ws=own)
        d_prep = sconv.make_desc(*shp[:10], None, True, prepared=True)
        d_plain = sconv.make_desc(*shp[:10], None, True)
        assert sconv.sconv_plan_name(d_prep) == plan and not _untuned(plan)
        assert _untuned(sconv.sconv_plan_name(d_plain))
        got = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, wprep=wp, ws=own)
        torch.cuda.synchronize()
        ref, scale = oracle.conv(x, w, 1, 1, 1, relu=True)
        assert (np.abs(got.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()
    finally:
        sconv.sconv_tune_reset()


@pytest.mark.parametrize("variant", ["rows", "tap", "quad", "wide", "gen", None])
@pytest.mark.parametrize("shp", [
    (2, 32, 19, 23, 70, 3, 3, 1, 1, 1, (2, 2, 2)),
    (2, 48, 14, 14, 192, 3, 3, 1, 1, 1, (2, 2, 2)),
    (1, 128, 28, 28, 128, 1, 1, 1, 0, 1, (2, 2, 2)),
    (2, 64, 30, 30, 96, 3, 3, 2, 1, 1, (2, 2, 2)),
])
def test_every_kernel_variant_on_the_same_input(device, monkeypatch, shp, variant):
    """The dispatch can be pinned; every variant that covers a shape must meet the same bars."""
    if variant is None:
        monkeypatch.delenv("SCONV_VARIANT", raising=False)
    else:
        monkeypatch.setenv("SCONV_VARIANT", variant)
    layer, x, w = _mk(110, shp)
    check_forward(layer, x, w, relu=True)
    check_pool_forward(layer, x, w)
    layer, x, w = _mk(111, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)


# 3x3 with whole 8-channel chunks, any stride and padding: the wide-granule matrix-core kernel
WIDE = [
    (2, 8, 19, 23, 70, 3, 3, 1, 1, 1, (2, 2, 2)),       # ragged filter block, rows cross images
    (1, 16, 28, 28, 32, 3, 3, 1, 1, 1, (2, 2, 2)),      # half-empty filter block
    (2, 24, 17, 30, 200, 3, 3, 1, 1, 1, (2, 2, 2)),     # two filters per lane, odd sizes
    (3, 64, 7, 7, 128, 3, 3, 1, 1, 1, (2, 2, 2)),       # 49-result planes: scalar stores
    (2, 64, 14, 14, 64, 3, 3, 1, 1, 2, (2, 2, 2)),      # grouped
    (1, 256, 9, 12, 256, 3, 3, 1, 1, 1, (2, 2, 2)),     # many chunks, channel slices
    (9, 16, 6, 5, 130, 3, 3, 1, 1, 1, (2, 2, 2)),       # several images per 64-row tile
    (2, 32, 19, 23, 70, 3, 3, 2, 1, 1, (2, 2, 2)),      # stride 2
    (1, 48, 28, 28, 160, 3, 3, 2, 1, 1, (2, 2, 2)),
    (2, 16, 20, 17, 40, 3, 3, 1, 0, 1, (2, 2, 2)),      # no padding
    (1, 16, 22, 22, 24, 3, 3, 3, 2, 1, (2, 2, 2)),      # stride 3, pad 2
    (1, 16, 3, 3, 5, 3, 3, 1, 1, 1, None),              # a single tile, mostly empty
]


# any kernel size, stride, padding and channel count: the general matrix-core kernel
GEN = [
    (1, 16, 21, 21, 20, 7, 7, 2, 3, 1, (2, 2, 2)),      # 7x7 / stride 2 / pad 3
    (2, 3, 31, 29, 70, 11, 11, 4, 2, 1, (2, 2, 2)),     # 3 channels, 11x11 / stride 4: L = 363, ragged chunk
    (1, 6, 14, 14, 16, 5, 5, 1, 0, 1, (2, 2, 2)),       # 5x5 without padding
    (2, 20, 12, 12, 50, 5, 5, 1, 2, 1, (2, 2, 2)),
    (1, 4, 9, 8, 6, 3, 2, 2, 1, 2, None),               # non-square kernel, grouped
    (2, 33, 17, 13, 130, 3, 3, 1, 1, 1, (2, 2, 2)),     # 3x3 with an odd channel count, two filters per lane
    (2, 48, 9, 11, 200, 1, 1, 2, 0, 1, None),           # 1x1 / stride 2
    (1, 2, 10, 11, 3, 5, 3, 3, 2, 1, None),             # stride 3, pad 2
    (1, 5, 3, 3, 4, 5, 5, 1, 2, 1, None),               # kernel larger than the map
    (3, 64, 7, 7, 128, 5, 5, 1, 2, 2, (2, 2, 2)),       # grouped, several images per 64-row tile
    (1, 192, 14, 14, 96, 5, 5, 1, 2, 1, (2, 2, 2)),     # L = 4800: many chunks
    (1, 1, 20, 20, 1, 15, 15, 1, 7, 1, None),           # largest kernel, one channel, one filter
]


@pytest.mark.parametrize("split", [None, "4,1", "8,2", "8,4"])
@pytest.mark.parametrize("shp", GEN)
def test_gen_variant(device, monkeypatch, shp, split):
    """The general matrix-core kernel pinned, with its own choice of column slices and with each
    split forced (the plan falls back to its own choice where a forced split does not apply)."""
    monkeypatch.setenv("SCONV_VARIANT", "gen")
    if split:
        monkeypatch.setenv("SCONV_GEN_SPLIT", split)
    layer, x, w = _mk(150, shp)
    d = sconv.desc_for(to_dev(x), to_dev(w), layer.stride, layer.pad, layer.groups, layer.pool, True)
    assert sconv.sconv_variant_name(d, False) == "gen"
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)
    if layer.pool:
        check_pool_forward(layer, x, w)
    layer, x, w = _mk(151, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    if layer.pool:
        check_pool_forward(layer, x, w, integer_exact=True)
    if split is None:
        for z in (0.0, 0.97, 1.0):
            layer, x, w = _mk(152, shp, z=z)
            check_forward(layer, x, w, relu=False)


QUAD = [s for s in SMALL if s[5:9] == (3, 3, 1, 1) and (s[1] // s[9]) % 16 == 0]


@pytest.mark.parametrize("shp", QUAD)
def test_quad_variant(device, monkeypatch, shp):
    """The default dispatch sends small launches to the vector kernel; the matrix-core 3x3 kernel
    is pinned here so that its ragged and small-map cases stay covered."""
    monkeypatch.setenv("SCONV_VARIANT", "quad")
    layer, x, w = _mk(116, shp)
    d = sconv.desc_for(to_dev(x), to_dev(w), layer.stride, layer.pad, layer.groups, layer.pool, True)
    assert sconv.sconv_variant_name(d, False) == "quad3x3"
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)
    check_pool_forward(layer, x, w)
    layer, x, w = _mk(117, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    check_pool_forward(layer, x, w, integer_exact=True)


@pytest.mark.parametrize("split", [None, "8,8", "8,2", "8,1"])
@pytest.mark.parametrize("shp", [
    (2, 32, 21, 56, 70, 3, 3, 1, 1, 1, None),           # three 7-row tiles, two column tiles, ragged filter block
    (1, 64, 9, 30, 64, 3, 3, 1, 1, 2, None),            # ragged last tile row, grouped
    (1, 128, 28, 28, 128, 3, 3, 1, 1, 1, None),
])
def test_quad_seven_row_tiles(device, monkeypatch, shp, split):
    """The 7-row tile geometry of the matrix-core 3x3 kernel, pinned, with every channel split."""
    monkeypatch.setenv("SCONV_VARIANT", "quad")
    monkeypatch.setenv("SCONV_QUAD_GEOM", "q32t7")
    if split:
        monkeypatch.setenv("SCONV_QUAD_SPLIT", split)
    layer, x, w = _mk(160, shp)
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)
    layer, x, w = _mk(161, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)


SPLIT = [
    (1, 512, 7, 7, 512, 3, 3, 1, 1, 1, (2, 2, 2)),      # the deep batch-1 layer the split is for
    (1, 64, 14, 14, 70, 3, 3, 1, 1, 1, (2, 2, 2)),      # ragged filter block
    (2, 96, 9, 11, 130, 3, 3, 1, 1, 2, (2, 2, 1)),      # grouped, 3 chunks per group: uneven ranges
    (1, 128, 13, 13, 64, 3, 3, 2, 1, 1, None),          # stride 2
]


@pytest.mark.parametrize("split", ["16,4,2", "8,8,4", "16,16,8", "8,1,2", "16,2,16"])
@pytest.mark.parametrize("shp", SPLIT)
def test_tap_channel_split_across_workgroups(device, monkeypatch, shp, split):
    """Partial sums of channel ranges through the scratch buffer, then the adding kernel with its
    ReLU / pooling epilogue: same bars as the one-kernel path (a split the shape has too few chunks
    for falls back to another kernel, which must match just the same)."""
    monkeypatch.setenv("SCONV_VARIANT", "tap")
    monkeypatch.setenv("SCONV_TAP_SPLIT", split)
    layer, x, w = _mk(180, shp)
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)
    if layer.pool:
        check_pool_forward(layer, x, w)
    layer, x, w = _mk(181, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    if layer.pool:
        check_pool_forward(layer, x, w, integer_exact=True)


@pytest.mark.parametrize("geom,split", [("q32k1", "8,4,2"), ("q32k1d", "16,4,4"), ("q32t7", "8,2,2"),
                                        ("q16k2", "16,2,4"), ("q32k2", "8,8,2")])
@pytest.mark.parametrize("shp", [
    (1, 64, 28, 30, 130, 3, 3, 1, 1, 1, None),          # wide map, ragged filter block
    (2, 128, 14, 14, 140, 3, 3, 1, 1, 2, None),         # map up to 14 wide, grouped
    (2, 64, 14, 13, 70, 3, 3, 1, 1, 1, (2, 2, 2)),      # fused pooling: plain tiles, pooled by the adding kernel
    (1, 48, 30, 58, 64, 3, 3, 1, 1, 1, (2, 2, 2)),      # the same on a wide map
])
def test_quad_channel_split_across_workgroups(device, monkeypatch, shp, geom, split):
    """The matrix-core 3x3 kernel with a tile's channels split over workgroups (a pinned plan: a
    geometry that does not fit the map's width falls back to another kernel, which must match too)."""
    monkeypatch.setenv("SCONV_VARIANT", "quad")
    monkeypatch.setenv("SCONV_QUAD_GEOM", geom)
    monkeypatch.setenv("SCONV_QUAD_SPLIT", split)
    layer, x, w = _mk(187, shp)
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)
    if layer.pool:
        check_pool_forward(layer, x, w)
    layer, x, w = _mk(188, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    if layer.pool:
        check_pool_forward(layer, x, w, integer_exact=True)


PW_SHAPES = [
    (2, 64, 9, 11, 70, 1, 1, 1, 0, 1, (2, 2, 2)),       # ragged filter block, odd plane size, ragged last tile
    (1, 128, 28, 28, 128, 1, 1, 1, 0, 1, (2, 2, 2)),
    (3, 256, 7, 7, 64, 1, 1, 1, 0, 2, (2, 2, 2)),       # grouped, plane smaller than a tile
    (1, 192, 30, 58, 40, 1, 1, 1, 0, 1, (2, 2, 2)),     # pooled tiles with ragged columns
    (2, 64, 5, 8, 64, 1, 1, 1, 0, 1, (2, 2, 2)),        # odd height: last row unpooled
]


@pytest.mark.parametrize("split", [None, "8,2", "16,4"])
@pytest.mark.parametrize("shp", PW_SHAPES)
def test_pointwise_dense_form(device, monkeypatch, shp, split):
    """The 1x1 matrix-core kernel without its zero tests: the same sums, and lanes that have no
    position must not leak into stored results (ragged tiles, pooled tiles with unused columns)."""
    monkeypatch.setenv("SCONV_PW_GEOM", "dense")
    if split:
        monkeypatch.setenv("SCONV_PW_SPLIT", split)
    layer, x, w = _mk(195, shp)
    d = sconv.desc_for(to_dev(x), to_dev(w), layer.stride, layer.pad, layer.groups, None, True)
    assert sconv.sconv_variant_name(d) == "quad1x1"
    check_forward(layer, x, w, relu=True)
    check_pool_forward(layer, x, w)
    layer, x, w = _mk(196, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    check_pool_forward(layer, x, w, integer_exact=True)


GEN_ANY_POOL = [
    (2, 20, 13, 13, 70, 3, 3, 1, 1, 1, (3, 3, 2)),      # overlapping 3x3 / stride 2 windows (7 per tile)
    (1, 48, 27, 27, 130, 5, 5, 1, 2, 2, (3, 3, 2)),     # grouped, two filters per lane possible
    (3, 16, 12, 10, 40, 3, 3, 1, 1, 1, (2, 3, 1)),      # 6-result windows, stride 1
    (1, 64, 16, 16, 64, 1, 1, 1, 0, 1, (4, 4, 4)),      # 1x1 convolution, 16-result windows
    (1, 8, 20, 20, 24, 3, 3, 2, 1, 1, (7, 7, 1)),       # 49-result windows: one per tile
    (2, 32, 9, 9, 64, 3, 3, 1, 1, 1, (2, 2, 1)),        # 2x2 windows of stride 1
]


@pytest.mark.parametrize("split", [None, "4,1", "8,2", "8,4"])
@pytest.mark.parametrize("shp", GEN_ANY_POOL)
def test_gen_fused_pooling_with_any_window(device, monkeypatch, shp, split):
    """Pooling windows other than 2x2 / stride 2 fused into the general matrix-core kernel: whole
    pooling windows per 64-row tile in PECR order, the maximum taken over a copy of the tile in LDS."""
    monkeypatch.setenv("SCONV_VARIANT", "gen")
    if split:
        monkeypatch.setenv("SCONV_GEN_SPLIT", split)
    layer, x, w = _mk(194, shp)
    d = sconv.desc_for(to_dev(x), to_dev(w), layer.stride, layer.pad, layer.groups, layer.pool, True)
    assert sconv.sconv_variant_name(d, True) == "gen"
    check_pool_forward(layer, x, w)
    layer, x, w = _mk(195, shp, integer=True)
    check_pool_forward(layer, x, w, integer_exact=True)
    layer, x, w = _mk(196, shp, z=1.0)
    check_pool_forward(layer, x, w)


GEN_SPLIT = [
    (1, 20, 11, 11, 50, 5, 5, 1, 0, 1, (2, 2, 2)),      # 500 columns: 8 chunks, the last one ragged
    (1, 480, 14, 14, 192, 1, 1, 1, 0, 1, (2, 2, 2)),    # 1x1 with a channel count off the 64 grid
    (2, 48, 7, 7, 130, 5, 5, 1, 2, 2, (2, 2, 1)),       # grouped, two filters per lane possible
    (1, 30, 9, 13, 40, 3, 4, 2, 1, 1, None),            # odd kernel, stride 2
]


@pytest.mark.parametrize("split", ["4,1,2", "8,2,4", "8,4,8", "4,4,2"])
@pytest.mark.parametrize("shp", GEN_SPLIT)
def test_gen_chunk_split_across_workgroups(device, monkeypatch, shp, split):
    """The general matrix-core kernel with its chunks split over workgroups: partial sums through
    the scratch buffer, epilogue (ReLU, any pooling window) in the adding kernel."""
    monkeypatch.setenv("SCONV_VARIANT", "gen")
    monkeypatch.setenv("SCONV_GEN_SPLIT", split)
    layer, x, w = _mk(183, shp)
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)
    if layer.pool:
        check_pool_forward(layer, x, w)
    layer, x, w = _mk(184, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    if layer.pool:
        check_pool_forward(layer, x, w, integer_exact=True)


def test_split_launches_on_two_streams_with_their_own_workspaces(device):
    """Workspaces are lent per stream: split launches of different layers enqueued on two streams at
    the same time, each stream with its own workspace, give what each gives alone."""
    shp_a = (1, 512, 7, 7, 512, 3, 3, 1, 1, 1, None)
    shp_b = (1, 256, 14, 14, 256, 3, 3, 1, 1, 1, None)
    la, xa, wa = _mk(185, shp_a)
    lb, xb, wb = _mk(186, shp_b)
    xad, wad, xbd, wbd = to_dev(xa), to_dev(wa), to_dev(xb), to_dev(wb)
    ref_a = sconv.sconv_forward(xad, wad, 1, 1, 1, relu=True)
    ref_b = sconv.sconv_forward(xbd, wbd, 1, 1, 1, relu=True)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    da = sconv.desc_for(xad, wad, 1, 1, 1, None, True)
    db = sconv.desc_for(xbd, wbd, 1, 1, 1, None, True)
    ws1 = torch.empty(sconv.sconv_workspace_size(da), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(sconv.sconv_workspace_size(db), dtype=torch.uint8, device="cuda")
    assert ws1.numel() > 0 and ws2.numel() > 0
    with torch.cuda.stream(s1):
        sconv.sconv_set_workspace(ws1)
    with torch.cuda.stream(s2):
        sconv.sconv_set_workspace(ws2)
    outs_a = [torch.empty_like(ref_a) for _ in range(20)]
    outs_b = [torch.empty_like(ref_b) for _ in range(20)]
    for oa, ob in zip(outs_a, outs_b):
        with torch.cuda.stream(s1):
            sconv.sconv_forward(xad, wad, 1, 1, 1, relu=True, out=oa)
        with torch.cuda.stream(s2):
            sconv.sconv_forward(xbd, wbd, 1, 1, 1, relu=True, out=ob)
    torch.cuda.synchronize()
    with torch.cuda.stream(s1):
        sconv.sconv_set_workspace(None)
    with torch.cuda.stream(s2):
        sconv.sconv_set_workspace(None)
    for oa, ob in zip(outs_a, outs_b):
        assert torch.equal(oa, ref_a) and torch.equal(ob, ref_b)
    check_forward(la, xa, wa, relu=True)


def test_a_workspace_that_is_too_small_or_absent_means_unsplit_plans(device):
    """A split plan needs the workspace lent for its stream: with one that is too small, and on a
    stream that has none (here one recording a graph), the launch runs unsplit and still matches."""
    shp = (1, 512, 7, 7, 512, 3, 3, 1, 1, 1, None)
    layer, x, w = _mk(182, shp)
    xd, wd = to_dev(x), to_dev(w)
    import oracle
    ref, scale = oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
    eager = sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True)   # default stream
    torch.cuda.synchronize()
    small = torch.empty(4096, dtype=torch.uint8, device="cuda")
    import conftest
    try:
        sconv.sconv_set_workspace(small)
        tiny_ws = sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True)
        torch.cuda.synchronize()
    finally:
        sconv.sconv_set_workspace(conftest._WORKSPACE)
    assert (np.abs(tiny_ws.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()
    out = torch.empty_like(eager)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True, out=out)
    for _ in range(3):
        out.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert (np.abs(out.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


def test_a_workspace_passed_with_the_call_splits_like_a_lent_one_and_none_means_unsplit(device):
    """sconv_forward_ws / sconv_pool_forward_ws: the workspace is an argument, nothing sticky.  With the
    same bytes as the lent one the launch plans the same split (bit-identical results); with none it
    runs unsplit; both meet the oracle's bar.  A lent workspace is ignored by these calls."""
    import oracle
    for shp, pool in (((1, 512, 7, 7, 512, 3, 3, 1, 1, 1, None), None),
                      ((2, 256, 14, 14, 128, 3, 3, 1, 1, 1, (2, 2, 2)), (2, 2, 2))):
        layer, x, w = _mk(187, shp)
        xd, wd = to_dev(x), to_dev(w)
        own = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        if pool:
            ref, scale = oracle.conv_pool(x, w, pool, 1, 1, 1)
            lent = sconv.sconv_pool_forward(xd, wd, pool, 1, 1, 1)
            given = sconv.sconv_pool_forward(xd, wd, pool, 1, 1, 1, ws=own)
            none = sconv.sconv_pool_forward(xd, wd, pool, 1, 1, 1, ws=None)
        else:
            ref, scale = oracle.conv(x, w, 1, 1, 1, relu=True)
            lent = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True)
            given = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, ws=own)
            none = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, ws=None)
        torch.cuda.synchronize()
        assert torch.equal(lent, given)
        for got in (given, none):
            assert (np.abs(got.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


@pytest.mark.parametrize("geom", ["gk1d", "gk2d", "gpk1d", "gpk2d"])
@pytest.mark.parametrize("shp", [
    (2, 20, 11, 11, 70, 5, 5, 1, 0, 1, (2, 2, 2)),
    (1, 30, 9, 13, 130, 3, 4, 2, 1, 1, (2, 2, 2)),
])
def test_gen_dense_candidates(device, monkeypatch, shp, geom):
    """The general matrix-core kernel without zero tests gives the same sums."""
    monkeypatch.setenv("SCONV_VARIANT", "gen")
    monkeypatch.setenv("SCONV_GEN_GEOM", geom)
    if geom.startswith("gp"):
        layer, x, w = _mk(190, shp)
        check_pool_forward(layer, x, w)
        layer, x, w = _mk(191, shp, integer=True)
        check_pool_forward(layer, x, w, integer_exact=True)
    else:
        layer, x, w = _mk(192, shp)
        check_forward(layer, x, w, relu=True)
        layer, x, w = _mk(193, shp, integer=True)
        check_forward(layer, x, w, relu=False, integer_exact=True)


@pytest.mark.parametrize("geom", ["q32t7d", "q32k1d", "q32k2d"])
@pytest.mark.parametrize("shp", [
    (2, 32, 21, 56, 70, 3, 3, 1, 1, 1, None),
    (1, 64, 9, 30, 64, 3, 3, 1, 1, 2, None),
    (1, 24, 28, 28, 130, 3, 3, 1, 1, 1, None),
])
def test_quad_dense_geometries(device, monkeypatch, shp, geom):
    """The matrix-core 3x3 tiles without zero tests (the dense form) give the same sums: the
    skipped products were zeros."""
    monkeypatch.setenv("SCONV_VARIANT", "quad")
    monkeypatch.setenv("SCONV_QUAD_GEOM", geom)
    layer, x, w = _mk(170, shp)
    check_forward(layer, x, w, relu=True)
    layer, x, w = _mk(171, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    layer, x, w = _mk(172, shp)
    x[:] = 0                      # an all-zero map still leaves through the whole-channel test
    check_forward(layer, x, w, relu=False)


@pytest.mark.parametrize("shp", WIDE)
def test_wide_variant(device, monkeypatch, shp):
    monkeypatch.setenv("SCONV_VARIANT", "wide")
    layer, x, w = _mk(112, shp)
    d = sconv.desc_for(to_dev(x), to_dev(w), layer.stride, layer.pad, layer.groups, layer.pool, True)
    assert sconv.sconv_variant_name(d, False) == "wide3x3"
    check_forward(layer, x, w, relu=True)
    check_forward(layer, x, w, relu=False)
    if layer.pool:
        assert sconv.sconv_variant_name(d, True) == "wide3x3"
        check_pool_forward(layer, x, w)
    layer, x, w = _mk(113, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)
    if layer.pool:
        check_pool_forward(layer, x, w, integer_exact=True)
    for z in (0.0, 0.97, 1.0):
        layer, x, w = _mk(114, shp, z=z)
        check_forward(layer, x, w, relu=False)


@pytest.mark.parametrize("shp", [SMALL[0], SMALL[1], SMALL[3], SMALL[7], SMALL[12], SMALL[17], SMALL[24]])
def test_unfused_pooling_kernel(device, shp):
    """ReLU + max pooling of a stored tensor is exact: equal to the oracle's pooling of the same
    fp32 values; and convolution followed by it meets the fused call's bar."""
    import oracle
    from parity import TOL
    layer, x, w = _mk(115, shp)
    xd, wd = to_dev(x), to_dev(w)
    conv = sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=False)
    got = sconv.sconv_maxpool(conv, x.shape, w.shape, layer.pool, layer.stride, layer.pad, layer.groups)
    torch.cuda.synchronize()
    conv_h = conv.cpu().numpy()
    want, _ = oracle.maxpool(np.maximum(conv_h, 0).astype(np.float64), layer.pool)
    assert np.array_equal(got.cpu().numpy().astype(np.float64), want)
    ref, scale = oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
    err = np.abs(got.cpu().numpy().astype(np.float64) - ref)
    assert (err <= TOL * scale).all()


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        R = S = int(rng.choice([1, 3, 3, 3, 5]))
        if rng.random() < 0.15:
            S = int(rng.choice([1, 2, 3]))
        groups = int(rng.choice([1, 1, 1, 2, 4]))
        Cg = int(rng.choice([3, 8, 16, 24, 32, 64, 128]))
        Kg = int(rng.integers(1, 140))
        stride = int(rng.choice([1, 1, 1, 2, 3]))
        pad = int(rng.integers(0, min(R, S)))
        H, W = int(rng.integers(max(R, 3), 36)), int(rng.integers(max(S, 3), 36))
        N = int(rng.integers(1, 4))
        OH, OW = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        if OH < 1 or OW < 1:
            continue
        pool = (2, 2, 2) if min(OH, OW) >= 2 and rng.random() < 0.8 else None
        out.append((N, Cg * groups, H, W, Kg * groups, R, S, stride, pad, groups, pool))
    return out


@pytest.mark.parametrize("shp", _random_shapes(40, 2024))
def test_random_shapes_through_the_default_dispatch(device, shp):
    """Seeded random shapes (kernel sizes, strides, paddings, groups, channel counts that do and do
    not fit the specialised kernels): whatever kernel the dispatch picks must meet the bars."""
    layer, x, w = _mk(140, shp, z=0.6)
    check_forward(layer, x, w, relu=True)
    if layer.pool:
        check_pool_forward(layer, x, w)
    layer, x, w = _mk(141, shp, integer=True)
    check_forward(layer, x, w, relu=False, integer_exact=True)


def _random_large_3x3(count, seed):
    """3x3 / stride 1 / pad 1 layers large enough for the rules that read the zero ratio and for the
    transposed-filter kernel (hundreds of tiles, 64-384 channels), small enough for the whole-tensor oracle."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        C = int(rng.choice([64, 96, 128, 192, 256, 384]))
        K = int(rng.choice([64, 100, 128, 192, 256]))
        H = int(rng.choice([7, 10, 14, 20, 28, 40]))
        W = H if rng.random() < 0.6 else int(rng.choice([7, 14, 20, 28]))
        N = int(rng.choice([4, 8, 16]))
        if 2.0 * N * K * H * W * C * 9 > 2e10 or N * H * W < 400:
            continue
        pool = (2, 2, 2) if rng.random() < 0.35 else None
        out.append((N, C, H, W, K, 3, 3, 1, 1, 1, pool))
    return out


@pytest.mark.parametrize("shp", _random_large_3x3(24, 99))
def test_random_large_layers_with_zero_ratio_hint_bias_and_explicit_workspace(device, shp):
    """Random 3x3 layers of benchmark size through every way of calling them: with the zero ratio reported in
    the descriptor (low, true and high - the hint may pick any variant, never a wrong result), with a bias,
    and with the workspace passed as an argument or withheld; whole tensors against the oracle."""
    import oracle
    rng = np.random.default_rng(sum(shp[:5]))
    z_true = float(rng.choice([0.45, 0.6, 0.75, 0.9]))
    layer, x, w = _mk(360, shp, z=z_true)
    b = (rng.standard_normal(shp[4]) * 0.3).astype(np.float32)
    xd, wd, bd = to_dev(x), to_dev(w), to_dev(b)
    own = torch.empty(48 << 20, dtype=torch.uint8, device="cuda")
    if layer.pool:
        ref, scale = oracle.conv_pool(x, w, layer.pool, 1, 1, 1)
        refb, scaleb = oracle.conv_pool_bias(x, w, b, layer.pool, 1, 1, 1)
        call = lambda **kw: sconv.sconv_pool_forward(xd, wd, layer.pool, 1, 1, 1, **kw)
    else:
        ref, scale = oracle.conv(x, w, 1, 1, 1, relu=True)
        refb, scaleb = oracle.conv_bias(x, w, b, 1, 1, 1, relu=True)
        call = lambda **kw: sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, **kw)
    outs = [(call(zero_ratio=zr), ref, scale, f"hint {zr}") for zr in (0.2, z_true, 0.97)]
    outs.append((call(ws=own), ref, scale, "own workspace"))
    outs.append((call(ws=None), ref, scale, "no workspace"))
    outs.append((call(bias=bd), refb, scaleb, "bias"))
    torch.cuda.synchronize()
    for got, r, sc, what in outs:
        err = np.abs(got.cpu().numpy().astype(np.float64) - r)
        assert (err <= 1e-4 * sc).all(), f"{what}: {int((err > 1e-4 * sc).sum())} outputs beyond the bar"


@pytest.mark.parametrize("shp", [
    (2, 32, 19, 23, 70, 3, 3, 1, 1, 1, (2, 2, 2)),      # tap / quad / wide / gen all apply
    (1, 128, 28, 28, 128, 1, 1, 1, 0, 1, (2, 2, 2)),     # quad1x1 / gen
    (2, 20, 12, 12, 50, 5, 5, 1, 2, 1, (2, 2, 2)),       # gen only
    (2, 64, 30, 30, 96, 3, 3, 2, 1, 1, None),            # stride 2: tap / wide / gen
    (1, 8, 40, 40, 16, 3, 3, 1, 1, 1, (7, 7, 3)),        # pooled: only the general kernel covers 7x7 windows
])
def test_tuned_plans_meet_the_same_bars(device, monkeypatch, shp):
    """sconv_tune picks whichever variant and decomposition measures fastest on the operands; the
    calls that follow launch it and must meet the parity bars; resetting brings the model back."""
    monkeypatch.delenv("SCONV_VARIANT", raising=False)
    sconv.sconv_tune_reset()
    try:
        layer, x, w = _mk(170, shp)
        xd, wd = to_dev(x), to_dev(w)
        d = sconv.desc_for(xd, wd, layer.stride, layer.pad, layer.groups, None, True)
        assert _untuned(sconv.sconv_plan_name(d))
        flush = torch.empty(8 << 20, dtype=torch.uint8, device="cuda") if shp[0] == 2 else None
        ms, plan = sconv.sconv_tune(xd, wd, layer.stride, layer.pad, layer.groups, None, relu=True, flush=flush)
        assert ms > 0 and plan == sconv.sconv_plan_name(d)
        assert plan.split("/")[0] == sconv.sconv_variant_name(d)
        check_forward(layer, x, w, relu=True)
        # relu=False is another descriptor: untouched by the tuning above
        d0 = sconv.desc_for(xd, wd, layer.stride, layer.pad, layer.groups, None, False)
        assert _untuned(sconv.sconv_plan_name(d0))
        check_forward(layer, x, w, relu=False)
        if layer.pool:
            dp = sconv.desc_for(xd, wd, layer.stride, layer.pad, layer.groups, layer.pool, True)
            ms, plan = sconv.sconv_tune(xd, wd, layer.stride, layer.pad, layer.groups, layer.pool)
            assert ms > 0 and plan == sconv.sconv_plan_name(dp, True)
            check_pool_forward(layer, x, w)
        layer, x, w = _mk(171, shp, integer=True)
        check_forward(layer, x, w, relu=True, integer_exact=False)
        check_forward(layer, x, w, relu=False, integer_exact=True)
        if layer.pool:
            check_pool_forward(layer, x, w, integer_exact=True)
    finally:
        sconv.sconv_tune_reset()
    assert _untuned(sconv.sconv_plan_name(d))


def test_tuned_plan_is_replayed_from_a_graph_and_yields_to_a_pinned_variant(device, monkeypatch):
    """A tuned descriptor's calls can be captured (tuning itself happened before the capture); and
    SCONV_VARIANT, when set, comes before the tuned table."""
    monkeypatch.delenv("SCONV_VARIANT", raising=False)
    sconv.sconv_tune_reset()
    try:
        shp = (2, 64, 14, 14, 128, 3, 3, 1, 1, 1, None)
        layer, x, w = _mk(175, shp)
        xd, wd = to_dev(x), to_dev(w)
        sconv.sconv_tune(xd, wd, 1, 1, 1, None, relu=True)
        d = sconv.desc_for(xd, wd, 1, 1, 1, None, True)
        assert not _untuned(sconv.sconv_plan_name(d))
        y = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        out = torch.empty_like(y)
        side_ws = torch.empty(sconv.sconv_workspace_size(d), dtype=torch.uint8, device="cuda")
        with torch.cuda.stream(side):
            # the tuned plan may be a split one: the capture stream needs a workspace of its own
            # (kept alive as long as the graph is replayed)
            sconv.sconv_set_workspace(side_ws)
            sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, out=out)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, out=out)
            sconv.sconv_set_workspace(None)
        torch.cuda.synchronize()
        for rep in range(3):
            _, xn, _ = _mk(176 + rep, shp)
            xd.copy_(torch.from_numpy(xn))
            out.fill_(-1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ref = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True)
            torch.cuda.synchronize()
            assert torch.equal(out, ref)
        monkeypatch.setenv("SCONV_VARIANT", "rows")
        assert sconv.sconv_variant_name(d) == "rows" and sconv.sconv_plan_name(d) == "rows/model"
        check_forward(layer, x, w, relu=True)
    finally:
        sconv.sconv_tune_reset()


def _random_prepared_3x3(count, seed):
    """3x3 / stride 1 / pad 1 layers over the ranges the static rules for prepared calls branch on: batch 1 to 32,
    maps 5 to 28 wide (7x7 and smaller whole-map tiles among them), 128 to 512 channels per group, groups, fused
    pooling; small enough for the whole-tensor oracle."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        G = int(rng.choice([1, 1, 1, 2, 4]))
        Cg = int(rng.choice([128, 160, 192, 256, 384, 512]))
        Kg = int(rng.choice([64, 96, 128, 192, 256]))
        H = int(rng.choice([5, 6, 7, 10, 14, 20, 28]))
        W = H if rng.random() < 0.7 else int(rng.choice([7, 14, 28]))
        N = int(rng.choice([1, 1, 2, 4, 8, 32]))
        if 2.0 * N * Kg * G * H * W * Cg * 9 > 1.2e10:
            continue
        pool = (2, 2, 2) if (rng.random() < 0.3 and H >= 6 and W >= 6) else None
        out.append((N, Cg * G, H, W, Kg * G, 3, 3, 1, 1, G, pool))
    return out


@pytest.mark.parametrize("shp", _random_prepared_3x3(20, 4711))
def test_random_layers_with_prepared_filters_through_the_static_rules(device, monkeypatch, shp):
    """Prepared calls through the default dispatch (no pins): with a workspace (small launches split over workgroups),
    without one, and with the zero ratio reported; whole tensors against the oracle."""
    import oracle
    monkeypatch.delenv("SCONV_VARIANT", raising=False)
    G = shp[9]
    layer, x, w = _mk(350, shp, z=0.8)
    xd, wd = to_dev(x), to_dev(w)
    wp = sconv.sconv_filter_prep(wd, groups=G)
    assert wp is not None
    own = torch.empty(48 << 20, dtype=torch.uint8, device="cuda")
    if layer.pool:
        ref, scale = oracle.conv_pool(x, w, layer.pool, 1, 1, G)
        call = lambda **kw: sconv.sconv_pool_forward(xd, wd, layer.pool, 1, 1, G, wprep=wp, **kw)
    else:
        ref, scale = oracle.conv(x, w, 1, 1, G, relu=True)
        call = lambda **kw: sconv.sconv_forward(xd, wd, 1, 1, G, relu=True, wprep=wp, **kw)
    outs = [(call(ws=own), "workspace"), (call(), "no workspace"), (call(ws=own, zero_ratio=0.8), "hint 0.8"),
            (call(ws=own, zero_ratio=0.3), "hint 0.3")]
    torch.cuda.synchronize()
    for got, what in outs:
        err = np.abs(got.cpu().numpy().astype(np.float64) - ref)
        assert (err <= 1e-4 * scale).all(), f"{what}: {int((err > 1e-4 * scale).sum())} outputs beyond the bar"


def test_exported_plans_are_replayed_after_import(device, monkeypatch):
    """Tune, export the table, forget it, import it: the same plans are launched without measuring again, and
    their results meet the oracle."""
    monkeypatch.delenv("SCONV_VARIANT", raising=False)
    sconv.sconv_tune_reset()
    try:
        cases = []
        for i, shp in enumerate([(4, 128, 14, 14, 128, 3, 3, 1, 1, 1, None), (2, 64, 28, 28, 64, 3, 3, 1, 1, 1, (2, 2, 2)),
                                 (8, 256, 14, 14, 64, 1, 1, 1, 0, 1, None)]):
            layer, x, w = _mk(360 + i, shp)
            xd, wd = to_dev(x), to_dev(w)
            _, plan = sconv.sconv_tune(xd, wd, shp[7], shp[8], shp[9], shp[10], relu=True)
            cases.append((layer, x, w, shp, plan))
        text = sconv.sconv_tune_export()
        assert len(text.splitlines()) == len(cases)
        sconv.sconv_tune_reset()
        for layer, x, w, shp, plan in cases:
            d = sconv.make_desc(*shp[:10], shp[10], True)
            assert _untuned(sconv.sconv_plan_name(d, shp[10] is not None))
        sconv.sconv_tune_import(text)
        for layer, x, w, shp, plan in cases:
            d = sconv.make_desc(*shp[:10], shp[10], True)
            assert sconv.sconv_plan_name(d, shp[10] is not None) == plan
            if layer.pool:
                check_pool_forward(layer, x, w)
            else:
                check_forward(layer, x, w, relu=True)
    finally:
        sconv.sconv_tune_reset()


def test_prepared_calls_keep_no_state_two_streams_and_a_graph(device, monkeypatch):
    """The ..._prep calls take everything as arguments: two streams, each with its own workspace and its own layer,
    run interleaved without touching each other; and such a call can be captured and replayed (no memset, no
    allocation, no host state)."""
    import oracle
    monkeypatch.delenv("SCONV_VARIANT", raising=False)
    shapes = [(4, 128, 14, 14, 192, 3, 3, 1, 1, 1, (2, 2, 2)), (1, 256, 14, 14, 256, 3, 3, 1, 1, 1, None)]
    cases = []
    for i, shp in enumerate(shapes):
        layer, x, w = _mk(340 + i, shp)
        xd, wd = to_dev(x), to_dev(w)
        cases.append((layer, x, w, xd, wd, sconv.sconv_filter_prep(wd), torch.empty(32 << 20, dtype=torch.uint8, device="cuda"),
                      torch.cuda.Stream()))
    torch.cuda.synchronize()
    outs = [None, None]
    for rep in range(4):                       # interleaved launches on the two streams
        for i, (layer, x, w, xd, wd, wp, ws, st) in enumerate(cases):
            with torch.cuda.stream(st):
                if layer.pool:
                    outs[i] = sconv.sconv_pool_forward(xd, wd, layer.pool, 1, 1, 1, wprep=wp, ws=ws, out=outs[i])
                else:
                    outs[i] = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, wprep=wp, ws=ws, out=outs[i])
    torch.cuda.synchronize()
    for i, (layer, x, w, *_rest) in enumerate(cases):
        if layer.pool:
            ref, scale = oracle.conv_pool(x, w, layer.pool, 1, 1, 1)
        else:
            ref, scale = oracle.conv(x, w, 1, 1, 1, relu=True)
        assert (np.abs(outs[i].cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()
    # capture the batch-1 layer (its plan splits the channels over workgroups: workspace traffic inside the graph)
    layer, x, w, xd, wd, wp, ws, st = cases[1]
    graph = torch.cuda.CUDAGraph()
    out = torch.empty_like(outs[1])
    with torch.cuda.stream(st):
        sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, wprep=wp, ws=ws, out=out)
        st.synchronize()
        with torch.cuda.graph(graph, stream=st):
            sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, wprep=wp, ws=ws, out=out)
    torch.cuda.synchronize()
    for rep in range(3):
        _, xn, _ = _mk(345 + rep, shapes[1])
        xd.copy_(torch.from_numpy(xn))
        out.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eager = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True, wprep=wp, ws=ws)
        torch.cuda.synchronize()
        assert torch.equal(out, eager)
        ref, scale = oracle.conv(xn, w, 1, 1, 1, relu=True)
        assert (np.abs(out.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


def test_small_launches_on_wide_maps_take_the_split_matrix_plan_when_a_workspace_is_lent(device, monkeypatch):
    """A 3x3 launch of 200-400 matrix-kernel tiles on a 28-wide map goes to quad3x3 with its channels
    split across workgroups when the stream has a workspace, and to the vector kernel when it has
    none; both meet the bars."""
    import conftest
    monkeypatch.delenv("SCONV_VARIANT", raising=False)
    sconv.sconv_tune_reset()
    shp = (4, 128, 28, 28, 256, 3, 3, 1, 1, 1, None)
    layer, x, w = _mk(188, shp)
    xd, wd = to_dev(x), to_dev(w)
    d = sconv.desc_for(xd, wd, 1, 1, 1, None, True)
    assert sconv.sconv_variant_name(d) == "quad3x3"
    check_forward(layer, x, w, relu=True)
    li, xi, wi = _mk(189, shp, integer=True)
    check_forward(li, xi, wi, relu=False, integer_exact=True)
    try:
        sconv.sconv_set_workspace(None)
        assert sconv.sconv_variant_name(d) == "tap3x3"
        check_forward(layer, x, w, relu=True)
    finally:
        sconv.sconv_set_workspace(conftest._WORKSPACE)


def test_a_tuned_split_plan_falls_back_when_its_workspace_is_taken_away(device, monkeypatch):
    """A plan tuned with a workspace may split its launch across workgroups; once the workspace
    is withdrawn the same descriptor must still run (unsplit) and meet the bar, and with the
    workspace back the tuned plan runs again."""
    import conftest
    import oracle
    monkeypatch.delenv("SCONV_VARIANT", raising=False)
    sconv.sconv_tune_reset()
    shp = (1, 512, 7, 7, 512, 3, 3, 1, 1, 1, None)
    layer, x, w = _mk(187, shp)
    xd, wd = to_dev(x), to_dev(w)
    ref, scale = oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
    try:
        # pin a split decomposition the way the tuner would remember it
        monkeypatch.setenv("SCONV_TAP_SPLIT", "16,16,8")
        monkeypatch.setenv("SCONV_VARIANT", "tap")
        with_ws = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True)
        torch.cuda.synchronize()
        sconv.sconv_set_workspace(None)
        without = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True)
        torch.cuda.synchronize()
        monkeypatch.delenv("SCONV_TAP_SPLIT")
        monkeypatch.delenv("SCONV_VARIANT")
        sconv.sconv_set_workspace(conftest._WORKSPACE)
        ms, plan = sconv.sconv_tune(xd, wd, 1, 1, 1, None, relu=True)
        tuned = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True)
        torch.cuda.synchronize()
        sconv.sconv_set_workspace(None)
        tuned_without = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=True)
        torch.cuda.synchronize()
    finally:
        sconv.sconv_set_workspace(conftest._WORKSPACE)
        sconv.sconv_tune_reset()
    for got in (with_ws, without, tuned, tuned_without):
        assert (np.abs(got.cpu().numpy().astype(np.float64) - ref) <= 1e-4 * scale).all()


def test_chained_layers_each_match_the_oracle_on_the_input_they_got(device):
    """Layers chained on the device (each consumes the previous one's output, zeros as ReLU and
    pooling left them): every layer is checked against the oracle applied to the very input the
    HIP path gave it, so errors cannot hide behind, or pile up across, layers."""
    import oracle
    from parity import TOL
    layers = [workloads.Layer("c0", C=32, H=20, W=20, K=64, R=3, S=3, pad=1, zero_ratio=0.6),
              workloads.Layer("c1", C=64, H=20, W=20, K=64, R=3, S=3, pad=1, pool=(2, 2, 2)),
              workloads.Layer("c2", C=64, H=10, W=10, K=48, R=1, S=1),
              workloads.Layer("c3", C=48, H=10, W=10, K=40, R=5, S=5, pad=2, pool=(2, 2, 2))]
    x, ws = workloads.make_chain_inputs(2, layers)
    cur = to_dev(x)
    for layer, w in zip(layers, ws):
        wd = to_dev(w)
        xin = cur.cpu().numpy()
        if layer.pool:
            y = sconv.sconv_pool_forward(cur, wd, layer.pool, layer.stride, layer.pad, layer.groups)
            ref, scale = oracle.conv_pool(xin, w, layer.pool, layer.stride, layer.pad, layer.groups)
        else:
            y = sconv.sconv_forward(cur, wd, layer.stride, layer.pad, layer.groups, relu=True)
            ref, scale = oracle.conv(xin, w, layer.stride, layer.pad, layer.groups, relu=True)
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
        assert got.shape == ref.shape
        assert (np.abs(got - ref) <= TOL * scale).all(), layer.name
        assert 0.3 < (got == 0).mean() < 0.999, "the chain should stay sparse but alive"
        cur = y


def test_outputs_are_overwritten_not_accumulated(device):
    shp = (1, 8, 12, 12, 16, 3, 3, 1, 1, 1, None)
    layer, x, w = _mk(108, shp)
    xd, wd = to_dev(x), to_dev(w)
    out = torch.full((1, 16, 12, 12), 1e9, dtype=torch.float32, device="cuda")
    sconv.sconv_forward(xd, wd, 1, 1, 1, relu=False, out=out)
    ref = sconv.sconv_forward(xd, wd, 1, 1, 1, relu=False)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_runs_on_a_side_stream(device):
    shp = (1, 8, 12, 12, 16, 3, 3, 1, 1, 1, None)
    layer, x, w = _mk(109, shp)
    xd, wd = to_dev(x), to_dev(w)
    ref = sconv.sconv_forward(xd, wd, 1, 1, 1)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        got = sconv.sconv_forward(xd, wd, 1, 1, 1)
    s.synchronize()
    assert torch.equal(got, ref)


def test_calls_can_be_captured_in_a_graph_and_replayed(device):
    """The library only enqueues on the caller's stream.  A captured sequence of its calls is
    replayed several times, with eager work and synchronisations in between, on fresh inputs
    written into the captured buffers; every replay must equal the eager result."""
    shapes = [(1, 64, 14, 14, 64, 3, 3, 1, 1, 1, (2, 2, 2)),      # tap3x3 (small launch)
              (1, 64, 14, 14, 128, 1, 1, 1, 0, 1, (2, 2, 2)),     # quad1x1
              (2, 16, 9, 9, 24, 3, 3, 2, 0, 1, None)]             # wide3x3
    cases = [_mk(120 + i, shp) for i, shp in enumerate(shapes)]
    bufs = []
    for layer, x, w in cases:
        xd, wd = to_dev(x), to_dev(w)
        y = sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True)
        z = sconv.sconv_pool_forward(xd, wd, layer.pool, layer.stride, layer.pad, layer.groups) if layer.pool else None
        bufs.append((layer, xd, wd, y, z))
    torch.cuda.synchronize()

    def step():
        for layer, xd, wd, y, z in bufs:
            sconv.sconv_forward(xd, wd, layer.stride, layer.pad, layer.groups, relu=True, out=y)
            if z is not None:
                sconv.sconv_pool_forward(xd, wd, layer.pool, layer.stride, layer.pad, layer.groups, out=z)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side_ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    with torch.cuda.stream(side):
        # the same plans as on the default stream (bitwise equal results) need a workspace here too
        sconv.sconv_set_workspace(side_ws)
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
        sconv.sconv_set_workspace(None)
    torch.cuda.synchronize()
    for rep in range(4):
        for i, (layer, xd, wd, y, z) in enumerate(bufs):          # fresh inputs in the captured buffers
            _, xn, _ = _mk(130 + 10 * rep + i, shapes[i])
            xd.copy_(torch.from_numpy(xn))
            y.fill_(-1.0)
            if z is not None:
                z.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [(y.clone(), None if z is None else z.clone()) for _, _, _, y, z in bufs]
        step()                                                     # the same work eagerly
        torch.cuda.synchronize()
        for (gy, gz), (_, _, _, y, z) in zip(got, bufs):
            assert torch.equal(gy, y)
            if z is not None:
                assert torch.equal(gz, z)
