"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and turns invalid descriptors into error codes before any GPU call."""
import ctypes
import os
import re

import pytest

import paper_1909_09927_amd as sconv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "sconv.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(sconv_[a-z_]+)\s*\(", text))
    assert {"sconv_encode", "sconv_forward", "sconv_pool_forward", "sconv_output_dims",
            "sconv_encode_sizes", "sconv_strerror", "sconv_variant_name", "sconv_maxpool", "sconv_tune",
            "sconv_tune_reset", "sconv_plan_name", "sconv_workspace_size", "sconv_set_workspace",
            "sconv_forward_ws", "sconv_pool_forward_ws", "sconv_env_refresh", "sconv_clear_workspaces",
            "sconv_forward_bias", "sconv_pool_forward_bias", "sconv_density",
            "sconv_forward_static", "sconv_pair_forward"} <= names
    L = sconv.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in sconv.h but not exported"


def test_header_is_self_contained_c_and_cpp(tmp_path):
    """include/sconv.h compiles on its own as C99 and as C++ (a C caller needs nothing else)."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "sconv.h")
    if shutil.which("gcc"):
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr],
                       check=True)
    if shutil.which("g++"):
        subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", hdr], check=True)


def test_a_plain_c_program_links_and_calls_the_library(tmp_path):
    """The boundary is a C ABI: a C99 program with only sconv.h links libsconv.so and calls it."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    src = tmp_path / "client.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "sconv.h"
int main(void) {
    sconv_desc_t d;
    memset(&d, 0, sizeof d);
    d.N = 2; d.C = 16; d.H = 28; d.W = 28; d.K = 32; d.R = 3; d.S = 3; d.stride = 1; d.pad = 1; d.groups = 1;
    d.pool_h = 2; d.pool_w = 2; d.pool_stride = 2;
    int32_t oh, ow, ph, pw;
    if (sconv_output_dims(&d, &oh, &ow, &ph, &pw) != SCONV_OK) return 1;
    d.stride = 0;
    int rc = sconv_forward(&d, (const float*)16, (const float*)16, (float*)16, NULL);
    printf("%d %d %d %d %d %s\n", oh, ow, ph, pw, rc, sconv_strerror(rc));
    return 0;
}
''')
    exe = tmp_path / "client"
    libdir = os.path.dirname(sconv.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-l:libsconv.so", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 5)
    assert out[:5] == ["28", "28", "14", "14", str(sconv.SCONV_EINVAL)] and "invalid" in out[5]


def test_output_dims_and_sizes():
    d = sconv.make_desc(2, 16, 28, 28, 32, 3, 3, 1, 1)
    assert sconv.sconv_output_dims(d) == (28, 28, 0, 0)
    assert sconv.sconv_encode_sizes(d, sconv.FMT_ECR) == (2 * 784, 144)
    d = sconv.make_desc(2, 16, 28, 28, 32, 3, 3, 1, 1, pool=(2, 2, 2))
    assert sconv.sconv_output_dims(d) == (28, 28, 14, 14)
    assert sconv.sconv_encode_sizes(d, sconv.FMT_PECR) == (2 * 14 * 14 * 4, 144)
    # figure sizes: 5x5 map, 3x3 kernel -> 3x3; 2x2 pooling stride 1 -> 2x2, 4 windows each
    d = sconv.make_desc(1, 1, 5, 5, 1, 3, 3, 1, 0, pool=(2, 2, 1))
    assert sconv.sconv_output_dims(d) == (3, 3, 2, 2)
    assert sconv.sconv_encode_sizes(d, sconv.FMT_PECR) == (16, 9)
    # floor: stride 2 on 56 with pad 1 -> 28; grouped L
    d = sconv.make_desc(1, 128, 56, 56, 128, 3, 3, 2, 1, groups=4)
    assert sconv.sconv_output_dims(d)[:2] == (28, 28)
    assert sconv.sconv_encode_sizes(d, sconv.FMT_ECR) == (4 * 784, 32 * 9)


BAD = [
    dict(N=0), dict(C=0), dict(H=-1), dict(K=0), dict(R=0), dict(S=0), dict(stride=0),
    dict(pad=-1), dict(groups=0), dict(groups=3), dict(K=30, groups=4), dict(pad=3), dict(flags=4),
    dict(H=1, pad=0),
]


@pytest.mark.parametrize("bad", BAD)
def test_invalid_descriptors_are_rejected_on_the_host(bad):
    base = dict(N=1, C=16, H=8, W=8, K=32, R=3, S=3, stride=1, pad=1, groups=1,
                pool_h=0, pool_w=0, pool_stride=0, flags=0)
    base.update(bad)
    d = sconv.Desc(**base)
    L = sconv.lib()
    oh, ow = ctypes.c_int32(), ctypes.c_int32()
    assert L.sconv_output_dims(ctypes.byref(d), ctypes.byref(oh), ctypes.byref(ow), None, None) == sconv.SCONV_EINVAL
    # non-null dummy pointers: the descriptor check must fire before anything touches them
    p = ctypes.c_void_p(16)
    assert L.sconv_forward(ctypes.byref(d), p, p, p, None) == sconv.SCONV_EINVAL
    assert L.sconv_encode(ctypes.byref(d), 0, p, p, p, p, None) == sconv.SCONV_EINVAL


def test_null_pointers_and_bad_pool_and_format():
    L = sconv.lib()
    d = sconv.make_desc(1, 16, 8, 8, 32, 3, 3, 1, 1)
    p = ctypes.c_void_p(16)
    assert L.sconv_forward(ctypes.byref(d), None, p, p, None) == sconv.SCONV_EINVAL
    assert L.sconv_forward(ctypes.byref(d), p, None, p, None) == sconv.SCONV_EINVAL
    assert L.sconv_forward(ctypes.byref(d), p, p, None, None) == sconv.SCONV_EINVAL
    assert L.sconv_forward(None, p, p, p, None) == sconv.SCONV_EINVAL
    # pooling call without / with an oversized pooling window
    assert L.sconv_pool_forward(ctypes.byref(d), p, p, p, None) == sconv.SCONV_EINVAL
    d2 = sconv.make_desc(1, 16, 8, 8, 32, 3, 3, 1, 1, pool=(9, 2, 2))
    assert L.sconv_pool_forward(ctypes.byref(d2), p, p, p, None) == sconv.SCONV_EINVAL
    d3 = sconv.make_desc(1, 16, 20, 20, 32, 3, 3, 1, 1, pool=(9, 9, 2))
    assert L.sconv_pool_forward(ctypes.byref(d3), p, p, p, None) == sconv.SCONV_EUNSUPPORTED
    assert L.sconv_maxpool(ctypes.byref(d), p, p, None) == sconv.SCONV_EINVAL
    rows, sl = ctypes.c_int64(), ctypes.c_int64()
    assert L.sconv_encode_sizes(ctypes.byref(d), 7, ctypes.byref(rows), ctypes.byref(sl)) == sconv.SCONV_EINVAL
    assert L.sconv_encode_sizes(ctypes.byref(d), sconv.FMT_PECR, ctypes.byref(rows), ctypes.byref(sl)) == sconv.SCONV_EINVAL


def test_too_large_tensors_are_unsupported():
    L = sconv.lib()
    p = ctypes.c_void_p(16)
    d = sconv.make_desc(4096, 1024, 1024, 1024, 8, 1, 1)
    assert L.sconv_forward(ctypes.byref(d), p, p, p, None) == sconv.SCONV_EUNSUPPORTED


def test_strerror_and_variant_name():
    assert sconv.strerror(0) == "success"
    assert "invalid" in sconv.strerror(sconv.SCONV_EINVAL)
    assert sconv.strerror(-99).startswith("unknown")
    assert sconv.sconv_variant_name(sconv.make_desc(1, 256, 56, 56, 64, 1, 1)) == "quad1x1"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 250, 56, 56, 64, 1, 1)) == "gen"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 16, 56, 56, 64, 5, 5, 1, 2)) == "gen"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 16, 56, 56, 64, 17, 17, 1, 2)) == "rows"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 16, 56, 56, 64, 5, 5, 1, 2, 1, (3, 3, 2)), True) == "gen"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 16, 56, 56, 64, 5, 5, 1, 2, 1, (9, 9, 2)), True) == "rows"
    assert sconv.sconv_variant_name(sconv.make_desc(32, 64, 56, 56, 64, 3, 3, 1, 1)) == "quad3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 64, 56, 56, 64, 3, 3, 1, 1)) == "tap3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 64, 56, 56, 64, 3, 3, 2, 1)) == "tap3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(32, 64, 56, 56, 64, 3, 3, 2, 1)) == "wide3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 64, 56, 56, 64, 3, 3, 2, 0)) == "wide3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 512, 7, 7, 512, 3, 3, 1, 1)) == "tap3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(32, 512, 7, 7, 512, 3, 3, 1, 1)) == "tap3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(32, 896, 14, 14, 896, 3, 3, 1, 1, 7)) == "wide3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(8, 512, 28, 28, 512, 3, 3, 1, 1)) == "tap3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(8, 256, 28, 28, 256, 3, 3, 1, 1)) == "quad3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(32, 512, 14, 14, 512, 3, 3, 1, 1, pool=(2, 2, 2)), True) == "tap3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(32, 256, 28, 28, 256, 3, 3, 1, 1, pool=(2, 2, 2)), True) == "quad3x3"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 64, 56, 56, 64, 5, 5, 1, 2)) == "gen"
    assert sconv.sconv_variant_name(sconv.make_desc(1, 64, 56, 56, 64, 3, 3, 1, 1, pool=(3, 3, 2)), True) == "gen"
    assert sconv.sconv_variant_name(sconv.Desc()) is None


def test_tuning_calls_validate_on_the_host():
    L = sconv.lib()
    d = sconv.make_desc(1, 16, 8, 8, 16, 3, 3, 1, 1)
    p = ctypes.c_void_p(16)
    assert L.sconv_tune(ctypes.byref(d), 0, None, p, p, None, 0, None, None) == sconv.SCONV_EINVAL
    assert L.sconv_tune(ctypes.byref(d), 0, p, p, p, p, 0, None, None) == sconv.SCONV_EINVAL    # scratch without a size
    assert L.sconv_tune(ctypes.byref(d), 0, p, p, p, None, 64, None, None) == sconv.SCONV_EINVAL
    bad = sconv.make_desc(1, 16, 8, 8, 16, 3, 3, 0, 1)
    assert L.sconv_tune(ctypes.byref(bad), 0, p, p, p, None, 0, None, None) == sconv.SCONV_EINVAL
    assert L.sconv_tune(ctypes.byref(d), 1, p, p, p, None, 0, None, None) == sconv.SCONV_EINVAL   # no pooling fields
    assert L.sconv_tune_reset() == 0
    assert sconv.sconv_plan_name(d).startswith("tap3x3/model")
    assert sconv.sconv_plan_name(sconv.make_desc(32, 64, 56, 56, 64, 3, 3, 1, 1)) == "quad3x3/model"
    buf = ctypes.create_string_buffer(4)
    assert L.sconv_plan_name(ctypes.byref(d), 0, buf, 4) == 0 and buf.value == b"tap"
    assert L.sconv_plan_name(ctypes.byref(d), 0, None, 4) == sconv.SCONV_EINVAL
    assert L.sconv_plan_name(ctypes.byref(bad), 0, buf, 4) == sconv.SCONV_EINVAL


def test_workspace_calls_validate_on_the_host():
    L = sconv.lib()
    n = ctypes.c_size_t(7)
    deep = sconv.make_desc(1, 512, 7, 7, 512, 3, 3, 1, 1)
    assert L.sconv_workspace_size(ctypes.byref(deep), 0, ctypes.byref(n)) == 0
    # sixteen slices of the convolution tensor + a transposed copy of the filters (+ 256 bytes of alignment)
    assert n.value == 16 * 512 * 49 * 4 + 512 * 512 * 9 * 4 + 256
    big = sconv.make_desc(32, 256, 56, 56, 256, 3, 3, 1, 1)
    assert L.sconv_workspace_size(ctypes.byref(big), 0, ctypes.byref(n)) == 0
    assert n.value == (64 << 20) + 256 * 256 * 9 * 4 + 256     # the partial sums are capped at 64 MiB
    odd = sconv.make_desc(1, 16, 40, 40, 8, 17, 17, 1, 2)     # only the window-row kernel covers it
    assert L.sconv_workspace_size(ctypes.byref(odd), 0, ctypes.byref(n)) == 0 and n.value == 0
    assert L.sconv_workspace_size(ctypes.byref(deep), 0, None) == sconv.SCONV_EINVAL
    assert L.sconv_workspace_size(ctypes.byref(sconv.Desc()), 0, ctypes.byref(n)) == sconv.SCONV_EINVAL
    assert L.sconv_workspace_size(ctypes.byref(deep), 1, ctypes.byref(n)) == sconv.SCONV_EINVAL   # no pooling fields
    assert L.sconv_set_workspace(ctypes.c_void_p(256), 0, None) == sconv.SCONV_EINVAL
    assert L.sconv_set_workspace(None, 4096, None) == sconv.SCONV_EINVAL
    assert L.sconv_set_workspace(ctypes.c_void_p(260), 4096, None) == sconv.SCONV_EINVAL          # not 16-byte aligned


def test_explicit_workspace_calls_validate_on_the_host():
    L = sconv.lib()
    d = sconv.make_desc(1, 16, 8, 8, 16, 3, 3, 1, 1, 1, (2, 2, 2))
    p = ctypes.c_void_p(4096)
    for fn in (L.sconv_forward_ws, L.sconv_pool_forward_ws):
        assert fn(ctypes.byref(d), None, p, p, None, 0, None) == sconv.SCONV_EINVAL          # null input
        assert fn(ctypes.byref(d), p, p, p, ctypes.c_void_p(4096), 0, None) == sconv.SCONV_EINVAL   # pointer, no bytes
        assert fn(ctypes.byref(d), p, p, p, None, 64, None) == sconv.SCONV_EINVAL            # bytes, no pointer
        assert fn(ctypes.byref(d), p, p, p, ctypes.c_void_p(4100), 64, None) == sconv.SCONV_EINVAL  # misaligned
    bad = sconv.make_desc(1, 16, 8, 8, 16, 3, 3, 0, 1, 1)
    assert L.sconv_forward_ws(ctypes.byref(bad), p, p, p, None, 0, None) == sconv.SCONV_EINVAL
    assert L.sconv_clear_workspaces() == sconv.SCONV_OK


def test_output_size_is_computed_in_64_bits():
    """H + 2*pad passes 2^31 with a large pad under a larger kernel: an error code, not an overflow."""
    L = sconv.lib()
    big = 2**31 - 1
    d = sconv.make_desc(1, 1, big, 4, 1, big, 3, 1, 2**30 + 5, 1)
    d.pad = 2**30 + 5
    oh, ow = ctypes.c_int32(), ctypes.c_int32()
    rc = L.sconv_output_dims(ctypes.byref(d), ctypes.byref(oh), ctypes.byref(ow), None, None)
    assert rc in (sconv.SCONV_EINVAL, sconv.SCONV_EUNSUPPORTED)


def test_environment_is_read_once_and_on_request(monkeypatch):
    """SCONV_VARIANT is a tuning aid the library reads once; sconv_env_refresh makes it look again."""
    d = sconv.make_desc(2, 64, 14, 14, 64, 3, 3, 1, 1, 1)
    os.environ.pop("SCONV_VARIANT", None)
    sconv.sconv_env_refresh()
    before = sconv.sconv_variant_name(d)
    os.environ["SCONV_VARIANT"] = "rows"
    try:
        assert sconv.sconv_variant_name(d) == before          # not looked at again
        sconv.sconv_env_refresh()
        assert sconv.sconv_variant_name(d) == "rows"
    finally:
        del os.environ["SCONV_VARIANT"]
        sconv.sconv_env_refresh()
    assert sconv.sconv_variant_name(d) == before


def test_density_calls_validate_on_the_host():
    L = sconv.lib()
    d = sconv.make_desc(1, 16, 8, 8, 16, 3, 3, 1, 1)
    p = ctypes.c_void_p(4096)
    assert L.sconv_density(ctypes.byref(d), None, p, None) == sconv.SCONV_EINVAL
    assert L.sconv_density(ctypes.byref(d), p, None, None) == sconv.SCONV_EINVAL
    assert L.sconv_density(ctypes.byref(d), p, ctypes.c_void_p(4100), None) == sconv.SCONV_EINVAL   # misaligned counts
    big = sconv.make_desc(32, 64, 56, 56, 64, 3, 3, 1, 1)
    assert sconv.sconv_variant_name(big) == "quad3x3"
    hinted = sconv.make_desc(32, 64, 56, 56, 64, 3, 3, 1, 1, zero_ratio=0.8)
    assert hinted.flags >> 8 == 1 + 203                                  # 1 + round(254 * 0.8)
    assert sconv.sconv_variant_name(hinted) == "tap3x3"                  # the hint moved the static choice
    assert sconv.sconv_variant_name(sconv.make_desc(32, 64, 56, 56, 64, 3, 3, 1, 1, zero_ratio=0.2)) == "quad3x3"
    bad = sconv.make_desc(32, 64, 56, 56, 64, 3, 3, 1, 1)
    bad.flags = 1 << 16                                                  # a bit no call defines
    assert sconv.sconv_variant_name(bad) is None
    with pytest.raises(ValueError):
        sconv.make_desc(1, 16, 8, 8, 16, 3, 3, 1, 1, zero_ratio=1.5)


def test_pair_call_validates_on_the_host():
    L = sconv.lib()
    d1 = sconv.make_desc(2, 1, 28, 28, 20, 5, 5, 1, 0, 1, (2, 2, 2))
    d2 = sconv.make_desc(2, 20, 12, 12, 50, 5, 5, 1, 0, 1, (2, 2, 2))
    p = ctypes.c_void_p(4096)
    call = lambda a, b, x=p, y=p: L.sconv_pair_forward(ctypes.byref(a), ctypes.byref(b), x, p, None, p, None, None, y, None)
    assert call(d1, d2, x=None) == sconv.SCONV_EINVAL
    assert call(d1, d2, y=None) == sconv.SCONV_EINVAL
    wrong = sconv.make_desc(2, 20, 11, 12, 50, 5, 5, 1, 0, 1, (2, 2, 2))     # not the first layer's output size
    assert call(d1, wrong) == sconv.SCONV_EINVAL
    grouped = sconv.make_desc(2, 20, 12, 12, 50, 5, 5, 1, 0, 2, (2, 2, 2))
    assert call(d1, grouped) == sconv.SCONV_EUNSUPPORTED
    big1 = sconv.make_desc(1, 64, 56, 56, 64, 3, 3, 1, 1)
    big2 = sconv.make_desc(1, 64, 56, 56, 64, 3, 3, 1, 1)
    assert call(big1, big2) == sconv.SCONV_EUNSUPPORTED


def test_binding_refuses_host_tensors():
    import torch
    x = torch.zeros(1, 2, 4, 4)
    w = torch.zeros(2, 2, 3, 3)
    with pytest.raises(TypeError):
        sconv.sconv_forward(x, w, pad=1)


def test_filter_prep_size_and_argument_checks():
    """Prepared filters: [group][block of 64 filters, even count][channel * 9 + tap][64] floats; only 3x3 /
    stride 1 / pad 1 layers with channels per group a multiple of 16 have a kernel that reads them."""
    L = sconv.lib()
    n = ctypes.c_size_t(123)
    d = sconv.make_desc(4, 512, 28, 28, 512, 3, 3, 1, 1)
    assert L.sconv_filter_prep_size(ctypes.byref(d), ctypes.byref(n)) == 0
    assert n.value == 512 * 512 * 9 * 4                       # 8 blocks of 64: nothing to pad
    d = sconv.make_desc(1, 128, 14, 14, 192, 3, 3, 1, 1, groups=2)   # 96 filters per group -> 2 blocks
    assert L.sconv_filter_prep_size(ctypes.byref(d), ctypes.byref(n)) == 0
    assert n.value == 2 * 2 * (64 * 9) * 64 * 4
    for other in (sconv.make_desc(1, 64, 14, 14, 64, 1, 1), sconv.make_desc(1, 64, 14, 14, 64, 3, 3, 2, 1),
                  sconv.make_desc(1, 24, 14, 14, 64, 3, 3, 1, 1), sconv.make_desc(1, 64, 14, 14, 64, 5, 5, 1, 2)):
        assert L.sconv_filter_prep_size(ctypes.byref(other), ctypes.byref(n)) == 0 and n.value == 0
        p = ctypes.c_void_p(256)
        assert L.sconv_filter_prep(ctypes.byref(other), p, p, 1 << 20, None) == sconv.SCONV_EUNSUPPORTED
    assert L.sconv_filter_prep_size(ctypes.byref(d), None) == sconv.SCONV_EINVAL
    p, odd = ctypes.c_void_p(256), ctypes.c_void_p(264)
    need = 2 * 2 * (64 * 9) * 64 * 4
    assert L.sconv_filter_prep(ctypes.byref(d), None, p, need, None) == sconv.SCONV_EINVAL
    assert L.sconv_filter_prep(ctypes.byref(d), p, None, need, None) == sconv.SCONV_EINVAL
    assert L.sconv_filter_prep(ctypes.byref(d), p, odd, need, None) == sconv.SCONV_EINVAL      # misaligned
    assert L.sconv_filter_prep(ctypes.byref(d), p, p, need - 1, None) == sconv.SCONV_EINVAL    # too small
    # the forward call: a half-given, misaligned or too small prepared copy is refused before any launch
    for f in (L.sconv_forward_prep, L.sconv_pool_forward_prep):
        dd = sconv.make_desc(1, 128, 14, 14, 192, 3, 3, 1, 1, groups=2, pool=(2, 2, 2))
        assert f(ctypes.byref(dd), p, p, p, 0, None, p, None, 0, None) == sconv.SCONV_EINVAL
        assert f(ctypes.byref(dd), p, p, None, need, None, p, None, 0, None) == sconv.SCONV_EINVAL
        assert f(ctypes.byref(dd), p, p, odd, need, None, p, None, 0, None) == sconv.SCONV_EINVAL
        assert f(ctypes.byref(dd), p, p, p, need - 256, None, p, None, 0, None) == sconv.SCONV_EINVAL
        assert f(ctypes.byref(dd), p, p, p, need, None, p, p, 0, None) == sconv.SCONV_EINVAL   # half-given workspace
        assert f(ctypes.byref(dd), None, p, p, need, None, p, None, 0, None) == sconv.SCONV_EINVAL


def test_tuned_plans_travel_as_text():
    """sconv_tune_export / sconv_tune_import: a plan line names the descriptor, the density class and whether
    filters come prepared; imported, later calls with that descriptor take it; malformed text imports nothing."""
    sconv.sconv_tune_reset()
    try:
        assert sconv.sconv_tune_export() == ""
        d = sconv.make_desc(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, None, True)
        key = "8 256 56 56 256 3 3 1 1 1 0 0 0 1 0 0 0"
        line = f"sconv-plan 1 {key} 2 1 q32t7d 8 4 0 0.24 quad3x3/q32t7d/8x4\n"
        sconv.sconv_tune_import(line)
        assert sconv.sconv_plan_name(d) == "quad3x3/q32t7d/8x4" and sconv.sconv_variant_name(d) == "quad3x3"
        # another batch size, another density class, prepared filters: other keys, still untuned
        assert "model" in sconv.sconv_plan_name(sconv.make_desc(4, 256, 56, 56, 256, 3, 3, 1, 1, 1, None, True))
        assert "model" in sconv.sconv_plan_name(sconv.make_desc(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, None, True, prepared=True))
        text = sconv.sconv_tune_export()
        assert text == line
        # a second entry (pooled layer, prepared filters, dense class 3) and a round trip through reset
        line2 = "sconv-plan 1 8 512 14 14 512 3 3 1 1 1 2 2 2 1 1 3 1 1 1 p2x14k1t 16 16 0 0.049 tap3x3/p2x14k1t/16x16\n"
        sconv.sconv_tune_import(line2)
        both = sconv.sconv_tune_export()
        assert sorted(both.splitlines()) == sorted((line + line2).splitlines())
        sconv.sconv_tune_reset()
        assert sconv.sconv_tune_export() == ""
        sconv.sconv_tune_import(both)
        dp = sconv.make_desc(8, 512, 14, 14, 512, 3, 3, 1, 1, 1, (2, 2, 2), True, zero_ratio=0.85, prepared=True)
        assert sconv.sconv_plan_name(dp, True) == "tap3x3/p2x14k1t/16x16"
        # nothing of a text with a bad line is taken: unknown geometry, bad counts, wrong version, short line
        sconv.sconv_tune_reset()
        for bad in (line.replace("q32t7d", "q99"), line.replace(" 8 4 0 0.24", " 8 3 0 0.24"),
                    line.replace("sconv-plan 1", "sconv-plan 2"), line2 + "sconv-plan 1 1 2 3\n",
                    line.replace(" 2 1 q32t7d", " 9 1 q32t7d"), "hello\n"):
            with pytest.raises(sconv.SconvError):
                sconv.sconv_tune_import(bad)
            assert sconv.sconv_tune_export() == ""
        L = sconv.lib()
        n = ctypes.c_size_t()
        sconv.sconv_tune_import(line)
        assert L.sconv_tune_export(None, 0, ctypes.byref(n)) == 0 and n.value == len(line) + 1
        small = ctypes.create_string_buffer(8)
        assert L.sconv_tune_export(small, 8, None) == sconv.SCONV_EINVAL
        assert L.sconv_tune_import(None) == sconv.SCONV_EINVAL
    finally:
        sconv.sconv_tune_reset()
