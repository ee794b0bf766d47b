"""Pins for the CPU oracle: every check here compares the oracle with something other than
itself: a brute-force loop on tiny inputs, a library routine on a special case, a closed form,
an invariant of the format, or a number the paper prints.  CPU only."""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# (N, C, H, W, K, R, S, stride, pad, groups)
SHAPES = [
    (1, 1, 5, 5, 1, 3, 3, 1, 0, 1),     # the paper's figure size
    (2, 3, 7, 6, 4, 3, 3, 1, 1, 1),
    (1, 4, 9, 8, 6, 3, 2, 2, 1, 2),     # non-square kernel, stride 2, groups
    (2, 6, 8, 8, 9, 1, 1, 1, 0, 3),     # 1x1 grouped
    (1, 2, 10, 11, 3, 5, 3, 3, 2, 1),   # stride 3, pad 2, non-dividing sizes
    (1, 8, 6, 6, 8, 3, 3, 1, 1, 8),     # depthwise
    (3, 5, 4, 9, 2, 2, 4, 2, 1, 1),
]


def _case(seed, shp, zero_ratio=0.6, integer=False):
    N, C, H, W, K, R, S, stride, pad, groups = shp
    return workloads.make_random_case(seed, N, C, H, W, K, R, S, stride, pad, groups,
                                      zero_ratio=zero_ratio, integer_valued=integer)


def _brute_conv(x, w, stride, pad, groups):
    """Seven nested Python loops over a padded copy, fp64 (tiny inputs only)."""
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    Kg = K // groups
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    OH = (H + 2 * pad - R) // stride + 1
    OW = (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, K, OH, OW), np.float64)
    for n in range(N):
        for k in range(K):
            g = k // Kg
            for oh in range(OH):
                for ow in range(OW):
                    t = 0.0
                    for c in range(Cg):
                        for r in range(R):
                            for s in range(S):
                                t += xp[n, g * Cg + c, oh * stride + r, ow * stride + s] * float(w[k, c, r, s])
                    y[n, k, oh, ow] = t
    return y


def _torch_conv(x, w, stride, pad, groups):
    return F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), None,
                    stride, pad, 1, groups).numpy()


# ---------------------------------------------------------------- convolution values

@pytest.mark.parametrize("shp", SHAPES[:5])
def test_conv_matches_brute_force(shp):
    layer, x, w = _case(11, shp)
    y, _ = oracle.conv(x, w, shp[7], shp[8], shp[9])
    ref = _brute_conv(x, w, shp[7], shp[8], shp[9])
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("shp", SHAPES)
def test_conv_matches_library_fp64(shp):
    layer, x, w = _case(12, shp)
    y, a = oracle.conv(x, w, shp[7], shp[8], shp[9])
    ref = _torch_conv(x, w, shp[7], shp[8], shp[9])
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-11)
    # the error scale is the same convolution of magnitudes
    ref_a = _torch_conv(np.abs(x), np.abs(w), shp[7], shp[8], shp[9])
    np.testing.assert_allclose(a, ref_a, rtol=1e-12, atol=1e-12)
    assert np.all(a >= np.abs(y) - 1e-12)


def test_conv_1x1_is_grouped_matrix_product():
    N, C, H, W, K, G = 2, 12, 5, 7, 8, 2
    layer, x, w = workloads.make_random_case(3, N, C, H, W, K, 1, 1, groups=G)
    y, _ = oracle.conv(x, w, groups=G)
    Cg, Kg = C // G, K // G
    for g in range(G):
        Wm = w[g * Kg:(g + 1) * Kg, :, 0, 0].astype(np.float64)            # [Kg, Cg]
        Xm = x[:, g * Cg:(g + 1) * Cg].reshape(N, Cg, H * W).astype(np.float64)
        ref = np.einsum("kc,ncp->nkp", Wm, Xm).reshape(N, Kg, H, W)
        np.testing.assert_allclose(y[:, g * Kg:(g + 1) * Kg], ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("r0,s0", [(0, 0), (1, 2), (2, 1)])
def test_delta_filter_shifts_the_map(r0, s0):
    # one filter tap equal to 1 at (r0, s0): y[oh, ow] = x padded at (oh - pad + r0, ow - pad + s0)
    N, C, H, W, R, S, pad = 1, 3, 6, 7, 3, 3, 1
    rng = np.random.default_rng(5)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = np.zeros((C, C, R, S), np.float32)
    for c in range(C):
        w[c, c, r0, s0] = 1.0
    y, _ = oracle.conv(x, w, 1, pad)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    ref = xp[:, :, r0:r0 + H, s0:s0 + W]
    np.testing.assert_array_equal(y, ref.astype(np.float64))


def test_ones_filter_is_box_sum():
    N, C, H, W, R, S = 1, 2, 8, 9, 3, 4
    rng = np.random.default_rng(6)
    x = rng.integers(0, 4, size=(N, C, H, W)).astype(np.float32)
    w = np.ones((1, C, R, S), np.float32)
    y, _ = oracle.conv(x, w)
    # box sums from a summed-area table
    sat = np.zeros((H + 1, W + 1))
    sat[1:, 1:] = x.sum(axis=1)[0].cumsum(0).cumsum(1)
    OH, OW = H - R + 1, W - S + 1
    ref = sat[R:R + OH, S:S + OW] - sat[:OH, S:S + OW] - sat[R:R + OH, :OW] + sat[:OH, :OW]
    np.testing.assert_array_equal(y[0, 0], ref)


def test_zero_input_gives_zero_and_linearity_in_filters():
    shp = SHAPES[2]
    layer, x, w = _case(21, shp)
    y0, a0 = oracle.conv(np.zeros_like(x), w, shp[7], shp[8], shp[9])
    assert not y0.any() and not a0.any()
    _, _, w2 = _case(22, shp)
    ya, _ = oracle.conv(x, w, shp[7], shp[8], shp[9])
    yb, _ = oracle.conv(x, w2, shp[7], shp[8], shp[9])
    # fp32 filter sum formed exactly in fp64 terms: compare against a convolution with 2*w (exact)
    y2, _ = oracle.conv(x, (2 * w).astype(np.float32), shp[7], shp[8], shp[9])
    np.testing.assert_allclose(y2, 2 * ya, rtol=0, atol=1e-12)
    assert np.abs(ya - yb).max() > 1e-3  # different filters do change the result


def test_integer_inputs_are_exact():
    for shp in SHAPES:
        layer, x, w = _case(31, shp, integer=True)
        y, a = oracle.conv(x, w, shp[7], shp[8], shp[9])
        ref = _torch_conv(x, w, shp[7], shp[8], shp[9])
        np.testing.assert_array_equal(y, ref)
        assert np.array_equal(y, np.round(y))


@pytest.mark.parametrize("shp", SHAPES)
def test_conv_at_points_matches_library(shp):
    layer, x, w = _case(13, shp)
    ref = _torch_conv(x, w, shp[7], shp[8], shp[9])
    ref_a = _torch_conv(np.abs(x), np.abs(w), shp[7], shp[8], shp[9])
    rng = np.random.default_rng(1)
    pts = np.stack([rng.integers(0, d, size=40) for d in ref.shape], axis=1)
    y, a = oracle.conv_at(x, w, pts, shp[7], shp[8], shp[9])
    np.testing.assert_allclose(y, ref[tuple(pts.T)], rtol=0, atol=1e-11)
    np.testing.assert_allclose(a, ref_a[tuple(pts.T)], rtol=1e-12, atol=1e-12)
    yr, _ = oracle.conv_at(x, w, pts, shp[7], shp[8], shp[9], relu=True)
    np.testing.assert_array_equal(yr, np.maximum(y, 0))


def test_relu_flag():
    shp = SHAPES[1]
    layer, x, w = _case(41, shp)
    y, _ = oracle.conv(x, w, shp[7], shp[8], shp[9])
    yr, _ = oracle.conv(x, w, shp[7], shp[8], shp[9], relu=True)
    assert (y < 0).any()
    np.testing.assert_array_equal(yr, np.maximum(y, 0))


# ---------------------------------------------------------------- pooling values

POOLS = [(2, 2, 2), (2, 2, 1), (3, 3, 2), (2, 3, 2), (1, 1, 1)]


@pytest.mark.parametrize("pool", POOLS)
@pytest.mark.parametrize("shp", [SHAPES[1], SHAPES[2], (1, 3, 11, 12, 5, 3, 3, 1, 1, 1)])
def test_conv_pool_matches_library(shp, pool):
    layer, x, w = _case(51, shp)
    OH = (shp[2] + 2 * shp[8] - shp[5]) // shp[7] + 1
    OW = (shp[3] + 2 * shp[8] - shp[6]) // shp[7] + 1
    if OH < pool[0] or OW < pool[1]:
        pytest.skip("pool window larger than conv output")
    z, sc = oracle.conv_pool(x, w, pool, shp[7], shp[8], shp[9])
    conv = torch.from_numpy(_torch_conv(x, w, shp[7], shp[8], shp[9]))
    ref = F.max_pool2d(torch.relu(conv), (pool[0], pool[1]), pool[2]).numpy()
    assert z.shape == ref.shape
    np.testing.assert_allclose(z, ref, rtol=0, atol=1e-11)
    # ReLU and max commute
    ref2 = torch.relu(F.max_pool2d(conv, (pool[0], pool[1]), pool[2])).numpy()
    np.testing.assert_allclose(z, ref2, rtol=0, atol=1e-11)
    # error scale = window maximum of the conv error scale
    a = torch.from_numpy(_torch_conv(np.abs(x), np.abs(w), shp[7], shp[8], shp[9]))
    ref_sc = F.max_pool2d(a, (pool[0], pool[1]), pool[2]).numpy()
    np.testing.assert_allclose(sc, ref_sc, rtol=1e-12, atol=1e-12)


def test_pool_1x1_equals_relu_conv():
    shp = SHAPES[1]
    layer, x, w = _case(52, shp)
    z, _ = oracle.conv_pool(x, w, (1, 1, 1), shp[7], shp[8], shp[9])
    y, _ = oracle.conv(x, w, shp[7], shp[8], shp[9], relu=True)
    np.testing.assert_array_equal(z, y)


def test_maxpool_brute_force():
    rng = np.random.default_rng(8)
    y = rng.standard_normal((2, 3, 7, 9))
    for pool in POOLS:
        z, _ = oracle.maxpool(y, pool)
        ph, pw, ps = pool
        PH, PW = (7 - ph) // ps + 1, (9 - pw) // ps + 1
        assert z.shape == (2, 3, PH, PW)
        for i, j in itertools.product(range(PH), range(PW)):
            win = y[:, :, i * ps:i * ps + ph, j * ps:j * ps + pw]
            np.testing.assert_array_equal(z[:, :, i, j], win.max(axis=(2, 3)))


# ---------------------------------------------------------------- encoding (ECR / PECR)

def _im2col_rows(x, R, S, stride, pad, groups):
    """Library im2col: rows[n, g, oh*OW+ow, c*R*S + r*S + s] via torch unfold."""
    N, C, H, W = x.shape
    Cg = C // groups
    cols = F.unfold(torch.from_numpy(x), (R, S), 1, pad, stride).numpy()  # [N, C*R*S, P]
    P = cols.shape[2]
    cols = cols.reshape(N, groups, Cg * R * S, P)
    return np.transpose(cols, (0, 1, 3, 2))  # [N, G, P, L]


@pytest.mark.parametrize("shp", SHAPES)
def test_ecr_round_trip_and_format_invariants(shp):
    N, C, H, W, K, R, S, stride, pad, groups = shp
    layer, x, w = _case(61, shp)
    values, index, count = oracle.encode(x, w.shape, oracle.FMT_ECR, stride, pad, groups)
    dense = _im2col_rows(x, R, S, stride, pad, groups).reshape(-1, (C // groups) * R * S)
    rows, L = dense.shape
    assert values.shape == (rows, L) and index.shape == (rows, L) and count.shape == (rows,)
    for r in range(rows):
        nz = np.flatnonzero(dense[r])
        c = count[r]
        if len(nz) == 0:
            assert c == -1          # Algorithm 1: marker for an empty window
            c = 0
        assert c == len(nz)         # brute-force nonzero count
        np.testing.assert_array_equal(index[r, :c], nz)           # scan order = ascending column
        np.testing.assert_array_equal(values[r, :c], dense[r, nz])
        assert not values[r, c:].any() and not index[r, c:].any()  # padding slots
        back = np.zeros(L, np.float32)
        back[index[r, :c]] = values[r, :c]
        np.testing.assert_array_equal(back, dense[r])               # scatter gives the im2col row


def test_ecr_tiny_by_hand():
    # 1 channel 3x3 map, 2x2 kernel, stride 1: four windows written out by hand.
    x = np.array([[[[0, 2, 0],
                    [3, 0, 0],
                    [0, 0, 5]]]], np.float32)
    values, index, count = oracle.encode(x, (1, 1, 2, 2), oracle.FMT_ECR)
    np.testing.assert_array_equal(count, [2, 1, 1, 1])
    np.testing.assert_array_equal(values, [[2, 3, 0, 0], [2, 0, 0, 0], [3, 0, 0, 0], [5, 0, 0, 0]])
    # positions inside the 2x2 filter, row-major: (0,1)=1 (1,0)=2 | (0,0)=0 | (0,0)=0 | (1,1)=3
    np.testing.assert_array_equal(index, [[1, 2, 0, 0], [0, 0, 0, 0], [0, 0, 0, 0], [3, 0, 0, 0]])
    # non-square kernel 1x3 on the top row: position = i*k_w + j
    values, index, count = oracle.encode(x[:, :, :1, :], (1, 1, 1, 3), oracle.FMT_ECR)
    np.testing.assert_array_equal(count, [1])
    np.testing.assert_array_equal(index[0], [1, 0, 0])
    # 3x1 kernel on the left column: x[1,0]=3 is tap i=1, j=0 -> 1*1+0
    values, index, count = oracle.encode(x[:, :, :, :1], (1, 1, 3, 1), oracle.FMT_ECR)
    np.testing.assert_array_equal(index[0], [1, 0, 0])
    # two channels: second channel's columns follow the first's (c*k_h*k_w + i*k_w + j)
    x2 = np.concatenate([x, x], axis=1)
    values, index, count = oracle.encode(x2, (1, 2, 2, 2), oracle.FMT_ECR)
    np.testing.assert_array_equal(count, [4, 2, 2, 2])
    np.testing.assert_array_equal(index[0], [1, 2, 5, 6, 0, 0, 0, 0])
    np.testing.assert_array_equal(values[0], [2, 3, 2, 3, 0, 0, 0, 0])


def test_nonzero_predicate():
    # IEEE "!= 0": both zeros are dropped, denormals and negative values are kept.
    x = np.array([[[[0.0, -0.0, 1e-42, -1.5]]]], np.float32)
    values, index, count = oracle.encode(x, (1, 1, 1, 4), oracle.FMT_ECR)
    assert count[0] == 2
    np.testing.assert_array_equal(index[0, :2], [2, 3])
    np.testing.assert_array_equal(values[0, :2], x[0, 0, 0, 2:])


def test_all_zero_and_all_dense_inputs():
    N, C, H, W, R, S, pad = 1, 2, 5, 6, 3, 3, 1
    w_shape = (1, C, R, S)
    z = np.zeros((N, C, H, W), np.float32)
    _, _, count = oracle.encode(z, w_shape, oracle.FMT_ECR, 1, pad)
    assert (count == -1).all()
    _, _, count = oracle.encode(z, w_shape, oracle.FMT_PECR, 1, pad, 1, (2, 2, 2))
    assert (count == 0).all()
    d = np.ones((N, C, H, W), np.float32)
    values, index, count = oracle.encode(d, w_shape, oracle.FMT_ECR, 1, pad)
    # in-bounds taps: rows 3 (interior) or 2 (border) times cols likewise, times C
    rows_in = np.array([2] + [3] * (H - 2) + [2])
    cols_in = np.array([2] + [3] * (W - 2) + [2])
    np.testing.assert_array_equal(count.reshape(H, W), C * np.outer(rows_in, cols_in))
    # interior window of a dense map: every column present, in order
    L = C * R * S
    r = 1 * W + 1
    np.testing.assert_array_equal(index[r], np.arange(L))


@pytest.mark.parametrize("shp", [SHAPES[1], SHAPES[2], SHAPES[4]])
def test_total_count_is_element_coverage(shp):
    """Sum of counts = sum over nonzero elements of the number of windows that contain them."""
    N, C, H, W, K, R, S, stride, pad, groups = shp
    layer, x, w = _case(62, shp)
    _, _, count = oracle.encode(x, w.shape, oracle.FMT_ECR, stride, pad, groups)
    OH = (H + 2 * pad - R) // stride + 1
    OW = (W + 2 * pad - S) // stride + 1
    cover_h = np.zeros(H, int)
    cover_w = np.zeros(W, int)
    for o in range(OH):
        for r in range(R):
            h = o * stride - pad + r
            if 0 <= h < H:
                cover_h[h] += 1
    for o in range(OW):
        for s in range(S):
            v = o * stride - pad + s
            if 0 <= v < W:
                cover_w[v] += 1
    cover = np.outer(cover_h, cover_w)
    expect = int(((x != 0) * cover[None, None]).sum())
    assert int(np.maximum(count, 0).sum()) == expect


@pytest.mark.parametrize("pool", [(2, 2, 2), (2, 2, 1), (3, 2, 2), (2, 2, 3)])
@pytest.mark.parametrize("shp", [SHAPES[0], SHAPES[1], SHAPES[2]])
def test_pecr_rows_are_ecr_rows_in_pooling_pack_order(shp, pool):
    N, C, H, W, K, R, S, stride, pad, groups = shp
    layer, x, w = _case(63, shp)
    ev, ei, ec = oracle.encode(x, w.shape, oracle.FMT_ECR, stride, pad, groups)
    pv, pi, pc = oracle.encode(x, w.shape, oracle.FMT_PECR, stride, pad, groups, pool)
    OH = (H + 2 * pad - R) // stride + 1
    OW = (W + 2 * pad - S) // stride + 1
    ph_, pw_, ps = pool
    PH, PW = (OH - ph_) // ps + 1, (OW - pw_) // ps + 1
    assert pv.shape[0] == N * groups * PH * PW * ph_ * pw_
    row = 0
    for n, g, a, b, py, px in itertools.product(range(N), range(groups), range(PH), range(PW),
                                                range(ph_), range(pw_)):
        e = ((n * groups + g) * OH + a * ps + py) * OW + b * ps + px
        np.testing.assert_array_equal(pv[row], ev[e])
        np.testing.assert_array_equal(pi[row], ei[e])
        assert pc[row] == max(ec[e], 0)          # PECR stores 0 where ECR stores -1
        row += 1


def test_pecr_duplicates_windows_when_pool_stride_is_smaller():
    # Fig. 7 geometry: 5x5 map, 3x3 kernel, 2x2 pooling, both strides 1: the centre conv window
    # (1,1) lies in all four pooling windows.
    rng = np.random.default_rng(9)
    x = rng.integers(1, 9, size=(1, 1, 5, 5)).astype(np.float32)  # distinct dense rows
    x[0, 0, 2, 2] = 77
    pv, pi, pc = oracle.encode(x, (1, 1, 3, 3), oracle.FMT_PECR, 1, 0, 1, (2, 2, 1))
    assert pv.shape == (2 * 2 * 4, 9)
    centre = x[0, 0, 1:4, 1:4].reshape(-1)
    hits = [r for r in range(16) if np.array_equal(pv[r], centre)]
    assert hits == [3, 6, 9, 12]   # (pw0:py1px1) (pw1:py1px0) (pw2:py0px1) (pw3:py0px0)


@pytest.mark.parametrize("shp", SHAPES)
def test_spmv_on_encoding_equals_dense_convolution(shp):
    """Algorithm 2 on Algorithm 1's output reproduces the plain convolution (zeros add nothing)."""
    N, C, H, W, K, R, S, stride, pad, groups = shp
    layer, x, w = _case(64, shp)
    values, index, count = oracle.encode(x, w.shape, oracle.FMT_ECR, stride, pad, groups)
    out = oracle.spmv(values, index, count, w, x.shape, stride, pad, groups)  # [rows, Kg]
    ref = _torch_conv(x, w, stride, pad, groups)                               # [N, K, OH, OW]
    OH, OW = ref.shape[2:]
    Kg = K // groups
    got = out.reshape(N, groups, OH * OW, Kg).transpose(0, 1, 3, 2).reshape(N, K, OH, OW)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-11)


def test_spmv_pecr_then_max_equals_fused_definition():
    shp, pool = SHAPES[1], (2, 2, 2)
    N, C, H, W, K, R, S, stride, pad, groups = shp
    layer, x, w = _case(65, shp)
    values, index, count = oracle.encode(x, w.shape, oracle.FMT_PECR, stride, pad, groups, pool)
    out = oracle.spmv(values, index, count, w, x.shape, stride, pad, groups, pool)
    z, _ = oracle.conv_pool(x, w, pool, stride, pad, groups)
    PH, PW = z.shape[2:]
    got = np.maximum(out, 0).reshape(N, PH * PW, 4, K).max(axis=2)      # max over the 4 threads
    got = got.transpose(0, 2, 1).reshape(N, K, PH, PW)
    np.testing.assert_allclose(got, z, rtol=0, atol=1e-11)


# ---------------------------------------------------------------- numbers the paper prints

def _read_kv(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = int(v)
    return out


def test_worked_example_operation_counts():
    g = _read_kv(os.path.join(GOLDEN, "opcount_example.txt"))
    # Eq. (1)/(2) for ONE block row of the 5x5 / 3x3 / stride-1 example: a 5-wide, 3-high strip
    mul, add = oracle.dense_op_counts(5, 3, 3, 3, 1)
    assert (mul, add) == (g["dense_mul"], g["dense_add"])
    # the figure's cell values did not survive; any strip whose three windows hold 3 + 4 + 3
    # nonzeros reproduces the printed totals (first window: 3 nonzeros)
    strip = np.array([[[[1, 0, 0, 2, 0],
                        [0, 3, 0, 0, 0],
                        [0, 0, 4, 5, 0]]]], np.float32)
    _, _, count = oracle.encode(strip, (1, 1, 3, 3), oracle.FMT_ECR)
    assert len(count) == g["windows"] and count[0] == g["first_window_nonzeros"]
    smul, sadd = oracle.sparse_op_counts(count)
    assert (smul, sadd) == (g["sparse_mul"], g["sparse_add"])
    assert round(100 * (1 - smul / mul)) == g["mul_saved_percent"]
    assert round(100 * (1 - sadd / add)) == g["add_saved_percent"]
    # whole-map form of Eq. (1)/(2): 3x3 windows of 9 taps
    assert oracle.dense_op_counts(5, 5, 3, 3, 1) == (81, 72)


def test_figure_geometry_and_eq3():
    with open(os.path.join(GOLDEN, "geometry_examples.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for name, i, k, cs, pw, ps, conv_out, pool_out, tpp, foot in rows:
        i, k, cs, pw, ps, conv_out, pool_out, tpp, foot = map(int, (i, k, cs, pw, ps, conv_out, pool_out, tpp, foot))
        pool = (pw, pw, ps) if pw else None
        shape = oracle.make_shape((1, 1, i, i), (1, 1, k, k), cs, 0, 1, pool)
        OH, OW, PH, PW = oracle.output_dims(shape)
        assert (OH, OW) == (conv_out, conv_out)
        if pw:
            assert (PH, PW) == (pool_out, pool_out)
            assert oracle.eq3_n_o(i, k, cs, pw, ps) == pool_out
            assert pw * pw == tpp
            assert k + cs * (pw - 1) == foot
            rows_, L = oracle.encode_sizes(shape, oracle.FMT_PECR)
            assert rows_ == tpp * pool_out ** 2      # p_w*p_h*n_o^2 threads per map (Section 6.3)
        rows_, L = oracle.encode_sizes(shape, oracle.FMT_ECR)
        assert rows_ == conv_out * conv_out and L == k * k


def test_eq3_equals_nested_floor_form_when_sizes_divide():
    for i, k, cs, pw, ps in itertools.product(range(5, 30), (1, 2, 3, 5), (1, 2, 3), (1, 2, 3), (1, 2, 3)):
        if (i - k) % cs:
            continue
        o = (i - k) // cs + 1
        if o < pw or (o - pw) % ps:
            continue
        shape = oracle.make_shape((1, 1, i, i), (1, 1, k, k), cs, 0, 1, (pw, pw, ps))
        assert oracle.eq3_n_o(i, k, cs, pw, ps) == oracle.output_dims(shape)[2] == (o - pw) // ps + 1


def test_expected_count_on_bernoulli_input():
    # E[count] = (1 - z) * taps for interior windows
    layer, x, w = workloads.make_layer_inputs(0, 0, 1)
    _, _, count = oracle.encode(x, w.shape, oracle.FMT_ECR, 1, 1)
    interior = count.reshape(28, 28)[1:-1, 1:-1]
    assert abs(interior.mean() / (16 * 9) - 0.3) < 0.01
    assert abs((x == 0).mean() - 0.7) < 0.01


# ---------------------------------------------------------------- bias (the layer's affine term)

@pytest.mark.parametrize("shp", SHAPES[:5])
def test_conv_bias_matches_brute_force_and_library(shp):
    """Bias is added to the plain sums before the ReLU: the 7-loop brute force plus b[k], the library's
    fp64 conv2d with its bias argument, and the error scale grown by |b[k]|."""
    layer, x, w = _case(41, shp)
    rng = np.random.default_rng(41)
    b = rng.standard_normal(shp[4]).astype(np.float32)
    y, a = oracle.conv_bias(x, w, b, shp[7], shp[8], shp[9], relu=False)
    ref = _brute_conv(x, w, shp[7], shp[8], shp[9]) + b.astype(np.float64)[None, :, None, None]
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)
    lib = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(),
                   shp[7], shp[8], 1, shp[9]).numpy()
    np.testing.assert_allclose(y, lib, rtol=0, atol=1e-11)
    _, a0 = oracle.conv(x, w, shp[7], shp[8], shp[9])
    np.testing.assert_allclose(a, a0 + np.abs(b.astype(np.float64))[None, :, None, None], rtol=0, atol=1e-12)
    yr, _ = oracle.conv_bias(x, w, b, shp[7], shp[8], shp[9], relu=True)
    np.testing.assert_array_equal(yr, np.maximum(y, 0.0))       # ReLU comes after the bias
    assert (yr != np.maximum(ref - b.astype(np.float64)[None, :, None, None], 0) + b[None, :, None, None]).any()


def test_bias_special_cases():
    """All-zero input: every output is its filter's bias (ReLU'd); zero bias: the plain convolution, bit
    for bit; a bias on one filter moves that filter's plane only."""
    shp = SHAPES[1]
    layer, x, w = _case(42, shp)
    b = np.array([0.5, -0.25, 2.0, -3.0], np.float32)
    y, a = oracle.conv_bias(np.zeros_like(x), w, b, shp[7], shp[8], shp[9], relu=True)
    np.testing.assert_array_equal(y, np.broadcast_to(np.maximum(b, 0).astype(np.float64)[None, :, None, None], y.shape))
    np.testing.assert_array_equal(a, np.broadcast_to(np.abs(b).astype(np.float64)[None, :, None, None], a.shape))
    y0, a0 = oracle.conv(x, w, shp[7], shp[8], shp[9])
    yz, az = oracle.conv_bias(x, w, np.zeros(4, np.float32), shp[7], shp[8], shp[9])
    np.testing.assert_array_equal(yz, y0)
    np.testing.assert_array_equal(az, a0)
    one = np.array([0, 0, 1.5, 0], np.float32)
    y1, _ = oracle.conv_bias(x, w, one, shp[7], shp[8], shp[9])
    np.testing.assert_array_equal(y1[:, [0, 1, 3]], y0[:, [0, 1, 3]])
    np.testing.assert_allclose(y1[:, 2], y0[:, 2] + 1.5, rtol=0, atol=1e-12)


@pytest.mark.parametrize("pool", [(2, 2, 2), (3, 3, 2)])
def test_conv_pool_bias_matches_library(pool):
    shp = (2, 3, 9, 10, 4, 3, 3, 1, 1, 1)
    layer, x, w = _case(43, shp)
    b = np.array([0.3, -0.7, 1.1, -0.1], np.float32)
    z, sc = oracle.conv_pool_bias(x, w, b, pool, shp[7], shp[8], shp[9])
    conv = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(),
                    shp[7], shp[8], 1, shp[9])
    ref = F.max_pool2d(torch.relu(conv), (pool[0], pool[1]), pool[2]).numpy()
    np.testing.assert_allclose(z, ref, rtol=0, atol=1e-11)
    assert (sc >= np.abs(b).min()).all()
