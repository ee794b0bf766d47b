"""Python binding of libsconv: zero-skipping direct convolution (+ fused max pooling) on MI355X.

Argument marshalling only: every step of the path runs in the HIP kernels behind the C ABI
declared in include/sconv.h.  PyTorch provides device memory and the current HIP stream.
There is no CPU fallback: without the built library every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsconv.so")

SCONV_RELU = 1
SCONV_PREPARED_FILTERS = 2
FMT_ECR = 0
FMT_PECR = 1
SCONV_OK, SCONV_EINVAL, SCONV_EUNSUPPORTED, SCONV_ELAUNCH, SCONV_ETOOLARGE = 0, -1, -2, -3, -4
STATIC_SCRATCH_BYTES = 16 << 20


class SconvError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class Desc(ctypes.Structure):
    """sconv_desc_t"""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride", "pad", "groups",
                 "pool_h", "pool_w", "pool_stride", "flags")]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; builds it first only when no built library exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        # torch first: its wheel carries its own HIP runtime, and the library must bind to the one the
        # process's streams and tensors come from (loading the library first would bring in the
        # system's copy as well, and launches on torch's streams then fail)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        L.sconv_output_dims.argtypes = [P(Desc), P(i32), P(i32), P(i32), P(i32)]
        L.sconv_encode_sizes.argtypes = [P(Desc), ctypes.c_int, P(i64), P(i64)]
        L.sconv_encode.argtypes = [P(Desc), ctypes.c_int, vp, vp, vp, vp, vp]
        L.sconv_forward.argtypes = [P(Desc), vp, vp, vp, vp]
        L.sconv_pool_forward.argtypes = [P(Desc), vp, vp, vp, vp]
        L.sconv_maxpool.argtypes = [P(Desc), vp, vp, vp]
        L.sconv_variant_name.argtypes = [P(Desc), ctypes.c_int]
        L.sconv_variant_name.restype = ctypes.c_char_p
        L.sconv_tune.argtypes = [P(Desc), ctypes.c_int, vp, vp, vp, vp, ctypes.c_size_t, vp, P(ctypes.c_float)]
        L.sconv_tune_reset.argtypes = []
        L.sconv_tune_export.argtypes = [ctypes.c_char_p, ctypes.c_size_t, P(ctypes.c_size_t)]
        L.sconv_tune_import.argtypes = [ctypes.c_char_p]
        L.sconv_plan_name.argtypes = [P(Desc), ctypes.c_int, ctypes.c_char_p, ctypes.c_int]
        L.sconv_strerror.argtypes = [ctypes.c_int]
        L.sconv_strerror.restype = ctypes.c_char_p
        L.sconv_workspace_size.argtypes = [P(Desc), ctypes.c_int, P(ctypes.c_size_t)]
        L.sconv_set_workspace.argtypes = [vp, ctypes.c_size_t, vp]
        L.sconv_clear_workspaces.argtypes = []
        L.sconv_env_refresh.argtypes = []
        L.sconv_forward_ws.argtypes = [P(Desc), vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.sconv_pool_forward_ws.argtypes = [P(Desc), vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.sconv_forward_static.argtypes = [P(Desc), vp, vp, vp, vp]
        L.sconv_forward_bias.argtypes = [P(Desc), vp, vp, vp, vp, vp]
        L.sconv_pool_forward_bias.argtypes = [P(Desc), vp, vp, vp, vp, vp]
        L.sconv_pair_forward.argtypes = [P(Desc), P(Desc), vp, vp, vp, vp, vp, vp, vp, vp]
        L.sconv_density.argtypes = [P(Desc), vp, vp, vp]
        sz = ctypes.c_size_t
        L.sconv_filter_prep_size.argtypes = [P(Desc), P(sz)]
        L.sconv_filter_prep.argtypes = [P(Desc), vp, vp, sz, vp]
        L.sconv_forward_prep.argtypes = [P(Desc), vp, vp, vp, sz, vp, vp, vp, sz, vp]
        L.sconv_pool_forward_prep.argtypes = [P(Desc), vp, vp, vp, sz, vp, vp, vp, sz, vp]
        L.sconv_tune_prep.argtypes = [P(Desc), ctypes.c_int, vp, vp, vp, sz, vp, vp, sz, vp, sz, vp,
                                      P(ctypes.c_float)]
        for f in ("sconv_output_dims", "sconv_encode_sizes", "sconv_encode", "sconv_forward",
                  "sconv_pool_forward", "sconv_maxpool", "sconv_tune", "sconv_tune_reset", "sconv_plan_name",
                  "sconv_workspace_size", "sconv_set_workspace", "sconv_clear_workspaces", "sconv_env_refresh",
                  "sconv_forward_ws", "sconv_pool_forward_ws", "sconv_forward_static", "sconv_forward_bias",
                  "sconv_pool_forward_bias", "sconv_pair_forward", "sconv_density", "sconv_filter_prep_size",
                  "sconv_filter_prep", "sconv_forward_prep", "sconv_pool_forward_prep", "sconv_tune_prep",
                  "sconv_tune_export", "sconv_tune_import"):
            getattr(L, f).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().sconv_strerror(code).decode()


def zero_ratio_flag(zero_ratio: Optional[float]) -> int:
    """SCONV_ZERO_RATIO(z): the optional density hint of a descriptor's flags (0 when None)."""
    if zero_ratio is None:
        return 0
    if not 0.0 <= zero_ratio <= 1.0:
        raise ValueError("zero_ratio must lie in [0, 1]")
    return (1 + int(zero_ratio * 254.0 + 0.5)) << 8


def make_desc(N, C, H, W, K, R, S, stride=1, pad=0, groups=1, pool: Optional[Tuple[int, int, int]] = None,
              relu: bool = False, zero_ratio: Optional[float] = None, prepared: bool = False) -> Desc:
    """prepared: SCONV_PREPARED_FILTERS, read by the two naming calls only."""
    ph, pw, ps = pool if pool is not None else (0, 0, 0)
    return Desc(N, C, H, W, K, R, S, stride, pad, groups, ph, pw, ps,
                (SCONV_RELU if relu else 0) | (SCONV_PREPARED_FILTERS if prepared else 0) |
                zero_ratio_flag(zero_ratio))


def desc_for(x, w, stride=1, pad=0, groups=1, pool=None, relu=False, zero_ratio=None, prepared=False) -> Desc:
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    if Cg * groups != C:
        raise ValueError("filter channel count does not match C / groups")
    return make_desc(N, C, H, W, K, R, S, stride, pad, groups, pool, relu, zero_ratio, prepared)


def sconv_output_dims(desc: Desc) -> Tuple[int, int, int, int]:
    v = [ctypes.c_int32() for _ in range(4)]
    rc = lib().sconv_output_dims(ctypes.byref(desc), *[ctypes.byref(t) for t in v])
    if rc:
        raise SconvError(rc, "sconv_output_dims")
    return tuple(t.value for t in v)


def sconv_encode_sizes(desc: Desc, fmt: int) -> Tuple[int, int]:
    rows, L = ctypes.c_int64(), ctypes.c_int64()
    rc = lib().sconv_encode_sizes(ctypes.byref(desc), fmt, ctypes.byref(rows), ctypes.byref(L))
    if rc:
        raise SconvError(rc, "sconv_encode_sizes")
    return rows.value, L.value


def sconv_variant_name(desc: Desc, pooled: bool = False) -> Optional[str]:
    s = lib().sconv_variant_name(ctypes.byref(desc), 1 if pooled else 0)
    return s.decode() if s is not None else None


def sconv_plan_name(desc: Desc, pooled: bool = False) -> str:
    buf = ctypes.create_string_buffer(64)
    rc = lib().sconv_plan_name(ctypes.byref(desc), 1 if pooled else 0, buf, len(buf))
    if rc:
        raise SconvError(rc, "sconv_plan_name")
    return buf.value.decode()


def sconv_tune_reset() -> None:
    lib().sconv_tune_reset()


def sconv_tune_export() -> str:
    """The plans sconv_tune has found so far, as text (one line per plan) for sconv_tune_import."""
    n = ctypes.c_size_t()
    lib().sconv_tune_export(None, 0, ctypes.byref(n))
    buf = ctypes.create_string_buffer(n.value)
    rc = lib().sconv_tune_export(buf, n.value, None)
    if rc:
        raise SconvError(rc, "sconv_tune_export")
    return buf.value.decode()


def sconv_tune_import(text: str) -> None:
    rc = lib().sconv_tune_import(text.encode())
    if rc:
        raise SconvError(rc, "sconv_tune_import")


def sconv_workspace_size(desc: Desc, pooled: bool = False) -> int:
    n = ctypes.c_size_t()
    rc = lib().sconv_workspace_size(ctypes.byref(desc), 1 if pooled else 0, ctypes.byref(n))
    if rc:
        raise ValueError(f"sconv_workspace_size: {strerror(rc)}")
    return int(n.value)


def sconv_set_workspace(ws) -> None:
    """Lends the device tensor `ws` (any dtype, contiguous) as the workspace of launches on torch's
    current stream; None withdraws it.  The caller keeps the tensor alive."""
    import torch
    if ws is None:
        rc = lib().sconv_set_workspace(None, 0, _stream())
    else:
        if not (isinstance(ws, torch.Tensor) and ws.is_cuda and ws.is_contiguous()):
            raise TypeError("ws must be a contiguous tensor in device memory")
        rc = lib().sconv_set_workspace(ws.data_ptr(), ws.numel() * ws.element_size(), _stream())
    if rc:
        raise RuntimeError(f"sconv_set_workspace: {strerror(rc)}")


def sconv_clear_workspaces() -> None:
    lib().sconv_clear_workspaces()


def sconv_env_refresh() -> None:
    """Makes the library read its SCONV_* tuning-aid environment variables again (it reads them once)."""
    lib().sconv_env_refresh()


def sconv_density(x, counts=None):
    """Enqueues the density probe on x (device, fp32, NCHW); returns the device tensor of two int64
    counts (examined, nonzero).  Reading it (e.g. zero_ratio_of) synchronises; the call itself does not."""
    import torch
    _check_dev(x, torch.float32, "x")
    N, C, H, W = x.shape
    desc = make_desc(N, C, H, W, C, 1, 1)
    if counts is None:
        counts = torch.empty(2, dtype=torch.int64, device=x.device)
    rc = lib().sconv_density(ctypes.byref(desc), x.data_ptr(), counts.data_ptr(), _stream())
    if rc:
        raise SconvError(rc, "sconv_density")
    return counts


def zero_ratio_of(counts) -> float:
    """Zero ratio from the probe's counts (copies them to the host: waits for the probe)."""
    seen, nonzero = (int(v) for v in counts.cpu())
    return 1.0 - nonzero / max(seen, 1)


def _ws_args(ws):
    """(pointer, bytes) of an explicit workspace: None -> (None, 0)."""
    import torch
    if ws is None:
        return None, 0
    if not (isinstance(ws, torch.Tensor) and ws.is_cuda and ws.is_contiguous()):
        raise TypeError("ws must be a contiguous tensor in device memory")
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _check_dev(t, dtype, what):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what} must be a contiguous {dtype} tensor in device memory")


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def sconv_encode(x, w_shape, fmt: int, stride=1, pad=0, groups=1, pool=None, out=None):
    """Format conversion alone; returns device tensors (values[rows,L], index[rows,L], count[rows]).
    out: an earlier result to write into instead of new tensors."""
    import torch
    _check_dev(x, torch.float32, "x")
    N, C, H, W = x.shape
    K, Cg, R, S = w_shape
    desc = make_desc(N, C, H, W, K, R, S, stride, pad, groups, pool)
    rows, L = sconv_encode_sizes(desc, fmt)
    if out is None:
        values = torch.empty((rows, L), dtype=torch.float32, device=x.device)
        index = torch.empty((rows, L), dtype=torch.int32, device=x.device)
        count = torch.empty((rows,), dtype=torch.int32, device=x.device)
    else:
        values, index, count = out
        _check_dev(values, torch.float32, "values")
        _check_dev(index, torch.int32, "index")
        _check_dev(count, torch.int32, "count")
        if tuple(values.shape) != (rows, L) or tuple(index.shape) != (rows, L) or tuple(count.shape) != (rows,):
            raise ValueError("out has the wrong shapes")
    rc = lib().sconv_encode(ctypes.byref(desc), fmt, x.data_ptr(), values.data_ptr(), index.data_ptr(),
                            count.data_ptr(), _stream())
    if rc:
        raise SconvError(rc, "sconv_encode")
    return values, index, count


_NO_WS = object()   # "no ws argument": the plain entry point (a lent workspace applies)


def sconv_filter_prep(w, groups=1, stride=1, pad=1, out=None):
    """The prepared (transposed) copy of the filters w[K,C/G,R,S] that the ..._prep calls read (a byte tensor
    in device memory), or None when no kernel reads the layout for such a layer."""
    import torch
    _check_dev(w, torch.float32, "w")
    K, Cg, R, S = w.shape
    desc = make_desc(1, Cg * groups, max(R, 8), max(S, 8), K, R, S, stride, pad, groups)
    n = ctypes.c_size_t()
    rc = lib().sconv_filter_prep_size(ctypes.byref(desc), ctypes.byref(n))
    if rc:
        raise SconvError(rc, "sconv_filter_prep_size")
    if n.value == 0:
        return None
    if out is None:
        out = torch.empty(n.value, dtype=torch.uint8, device=w.device)
    rc = lib().sconv_filter_prep(ctypes.byref(desc), w.data_ptr(), out.data_ptr(), out.numel(), _stream())
    if rc:
        raise SconvError(rc, "sconv_filter_prep")
    return out


def _opt_ptr(t):
    return (t.data_ptr(), t.numel() * t.element_size()) if t is not None else (None, 0)


def sconv_forward(x, w, stride=1, pad=0, groups=1, relu=False, out=None, ws=_NO_WS, bias=None, zero_ratio=None,
                  wprep=None):
    """Sparse convolution; returns y[N,K,OH,OW] (device, fp32).  ws: a device tensor (or None) passed as
    this call's workspace through sconv_forward_ws; left out, sconv_forward runs.  bias: a device tensor
    [K] added before the ReLU (sconv_forward_bias; not together with ws).  zero_ratio: the map's zero
    ratio if known (a hint for the choice of kernel, carried in the descriptor's flags).  wprep: the prepared
    copy of w (sconv_filter_prep); with it sconv_forward_prep runs, taking bias and ws (None when left out:
    a lent workspace does not apply) as arguments of the call."""
    import torch
    _check_dev(x, torch.float32, "x")
    _check_dev(w, torch.float32, "w")
    desc = desc_for(x, w, stride, pad, groups, None, relu, zero_ratio)
    OH, OW, _, _ = sconv_output_dims(desc)
    if out is None:
        out = torch.empty((desc.N, desc.K, OH, OW), dtype=torch.float32, device=x.device)
    else:
        _check_dev(out, torch.float32, "out")
        if tuple(out.shape) != (desc.N, desc.K, OH, OW):
            raise ValueError("out has the wrong shape")
    if wprep is not None:
        if bias is not None:
            _check_dev(bias, torch.float32, "bias")
        wp, wb = _ws_args(None if ws is _NO_WS else ws)
        pp, pb = _opt_ptr(wprep)
        rc = lib().sconv_forward_prep(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), pp, pb,
                                      bias.data_ptr() if bias is not None else None, out.data_ptr(), wp, wb,
                                      _stream())
    elif bias is not None:
        _check_dev(bias, torch.float32, "bias")
        if ws is not _NO_WS or tuple(bias.shape) != (desc.K,):
            raise ValueError("bias must be [K] and cannot be combined with an explicit workspace")
        rc = lib().sconv_forward_bias(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), bias.data_ptr(),
                                      out.data_ptr(), _stream())
    elif ws is _NO_WS:
        rc = lib().sconv_forward(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), out.data_ptr(), _stream())
    else:
        wp, wb = _ws_args(ws)
        rc = lib().sconv_forward_ws(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), out.data_ptr(), wp, wb,
                                    _stream())
    if rc:
        raise SconvError(rc, "sconv_forward")
    return out


def sconv_forward_static(x, w, stride=1, pad=0, groups=1, relu=False, out=None):
    """sconv_forward with the library's static scratch as workspace (allocates nothing itself: pass
    `out` to keep the whole call allocation-free); raises SconvError(SCONV_ETOOLARGE) beyond its limit."""
    import torch
    _check_dev(x, torch.float32, "x")
    _check_dev(w, torch.float32, "w")
    desc = desc_for(x, w, stride, pad, groups, None, relu)
    OH, OW, _, _ = sconv_output_dims(desc)
    if out is None:
        out = torch.empty((desc.N, desc.K, OH, OW), dtype=torch.float32, device=x.device)
    else:
        _check_dev(out, torch.float32, "out")
        if tuple(out.shape) != (desc.N, desc.K, OH, OW):
            raise ValueError("out has the wrong shape")
    rc = lib().sconv_forward_static(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), out.data_ptr(), _stream())
    if rc:
        raise SconvError(rc, "sconv_forward_static")
    return out


def sconv_pair_forward(x, w1, w2, first, second, bias1=None, bias2=None, keep_mid=False):
    """Two layers in one launch, the first layer's output handed over in LDS.  first / second: dicts with
    stride, pad, pool (None or (p_h, p_w, p_s)) and relu.  Returns (y, mid or None)."""
    import torch
    for t, name in ((x, "x"), (w1, "w1"), (w2, "w2")):
        _check_dev(t, torch.float32, name)
    d1 = desc_for(x, w1, first.get("stride", 1), first.get("pad", 0), 1, first.get("pool"), first.get("relu", True))
    oh1, ow1, ph1, pw1 = sconv_output_dims(d1)
    mh, mw = (ph1, pw1) if first.get("pool") else (oh1, ow1)
    d2 = make_desc(d1.N, d1.K, mh, mw, w2.shape[0], w2.shape[2], w2.shape[3], second.get("stride", 1),
                   second.get("pad", 0), 1, second.get("pool"), second.get("relu", True))
    oh2, ow2, ph2, pw2 = sconv_output_dims(d2)
    yh, yw = (ph2, pw2) if second.get("pool") else (oh2, ow2)
    y = torch.empty((d1.N, d2.K, yh, yw), dtype=torch.float32, device=x.device)
    mid = torch.empty((d1.N, d1.K, mh, mw), dtype=torch.float32, device=x.device) if keep_mid else None
    for b, name in ((bias1, "bias1"), (bias2, "bias2")):
        if b is not None:
            _check_dev(b, torch.float32, name)
    rc = lib().sconv_pair_forward(ctypes.byref(d1), ctypes.byref(d2), x.data_ptr(), w1.data_ptr(),
                                  bias1.data_ptr() if bias1 is not None else None, w2.data_ptr(),
                                  bias2.data_ptr() if bias2 is not None else None,
                                  mid.data_ptr() if mid is not None else None, y.data_ptr(), _stream())
    if rc:
        raise SconvError(rc, "sconv_pair_forward")
    return y, mid


def sconv_maxpool(conv, x_shape, w_shape, pool, stride=1, pad=0, groups=1, out=None):
    """ReLU + max pooling of a stored convolution tensor conv[N,K,OH,OW]; returns y[N,K,PH,PW]."""
    import torch
    _check_dev(conv, torch.float32, "conv")
    N, C, H, W = x_shape
    K, Cg, R, S = w_shape
    desc = make_desc(N, C, H, W, K, R, S, stride, pad, groups, pool, True)
    OH, OW, PH, PW = sconv_output_dims(desc)
    if tuple(conv.shape) != (N, K, OH, OW):
        raise ValueError("conv has the wrong shape")
    if out is None:
        out = torch.empty((N, K, PH, PW), dtype=torch.float32, device=conv.device)
    else:
        _check_dev(out, torch.float32, "out")
        if tuple(out.shape) != (N, K, PH, PW):
            raise ValueError("out has the wrong shape")
    rc = lib().sconv_maxpool(ctypes.byref(desc), conv.data_ptr(), out.data_ptr(), _stream())
    if rc:
        raise SconvError(rc, "sconv_maxpool")
    return out


def sconv_pool_forward(x, w, pool, stride=1, pad=0, groups=1, out=None, ws=_NO_WS, bias=None, zero_ratio=None,
                       wprep=None):
    """Sparse convolution + ReLU + max pooling in one pass; returns y[N,K,PH,PW] (device, fp32).
    ws, bias, zero_ratio, wprep: as in sconv_forward."""
    import torch
    _check_dev(x, torch.float32, "x")
    _check_dev(w, torch.float32, "w")
    desc = desc_for(x, w, stride, pad, groups, pool, True, zero_ratio)
    _, _, PH, PW = sconv_output_dims(desc)
    if out is None:
        out = torch.empty((desc.N, desc.K, PH, PW), dtype=torch.float32, device=x.device)
    else:
        _check_dev(out, torch.float32, "out")
        if tuple(out.shape) != (desc.N, desc.K, PH, PW):
            raise ValueError("out has the wrong shape")
    if wprep is not None:
        if bias is not None:
            _check_dev(bias, torch.float32, "bias")
        wp, wb = _ws_args(None if ws is _NO_WS else ws)
        pp, pb = _opt_ptr(wprep)
        rc = lib().sconv_pool_forward_prep(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), pp, pb,
                                           bias.data_ptr() if bias is not None else None, out.data_ptr(), wp, wb,
                                           _stream())
    elif bias is not None:
        _check_dev(bias, torch.float32, "bias")
        if ws is not _NO_WS or tuple(bias.shape) != (desc.K,):
            raise ValueError("bias must be [K] and cannot be combined with an explicit workspace")
        rc = lib().sconv_pool_forward_bias(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), bias.data_ptr(),
                                           out.data_ptr(), _stream())
    elif ws is _NO_WS:
        rc = lib().sconv_pool_forward(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), out.data_ptr(), _stream())
    else:
        wp, wb = _ws_args(ws)
        rc = lib().sconv_pool_forward_ws(ctypes.byref(desc), x.data_ptr(), w.data_ptr(), out.data_ptr(), wp, wb,
                                         _stream())
    if rc:
        raise SconvError(rc, "sconv_pool_forward")
    return out


def sconv_tune(x, w, stride=1, pad=0, groups=1, pool=None, relu=False, out=None, flush=None, zero_ratio=None,
               wprep=None, ws=None):
    """Times every kernel variant and decomposition covering this call on x and w (synchronises)
    and makes later identical calls use the fastest.  pool=None tunes sconv_forward (with this
    relu flag), else sconv_pool_forward.  flush: a device tensor the library may overwrite to evict
    the caches before every timed launch (cold ranking); None ranks cache-warm.  wprep: tune the calls that
    bring this prepared copy of w (sconv_tune_prep, with ws as its workspace argument).
    Returns (milliseconds of the chosen plan, plan name)."""
    import torch
    _check_dev(x, torch.float32, "x")
    _check_dev(w, torch.float32, "w")
    pooled = pool is not None
    desc = desc_for(x, w, stride, pad, groups, pool, True if pooled else relu, zero_ratio)
    OH, OW, PH, PW = sconv_output_dims(desc)
    shape = (desc.N, desc.K, PH, PW) if pooled else (desc.N, desc.K, OH, OW)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    else:
        _check_dev(out, torch.float32, "out")
        if tuple(out.shape) != shape:
            raise ValueError("out has the wrong shape")
    ms = ctypes.c_float(0.0)
    fptr, fbytes = (None, 0)
    if flush is not None:
        if not (isinstance(flush, torch.Tensor) and flush.is_cuda and flush.is_contiguous()):
            raise TypeError("flush must be a contiguous tensor in device memory")
        fptr, fbytes = flush.data_ptr(), flush.numel() * flush.element_size()
    if wprep is not None:
        wp, wb = _ws_args(ws)
        pp, pb = _opt_ptr(wprep)
        rc = lib().sconv_tune_prep(ctypes.byref(desc), 1 if pooled else 0, x.data_ptr(), w.data_ptr(), pp, pb,
                                   out.data_ptr(), wp, wb, fptr, fbytes, _stream(), ctypes.byref(ms))
        desc.flags |= SCONV_PREPARED_FILTERS
    else:
        rc = lib().sconv_tune(ctypes.byref(desc), 1 if pooled else 0, x.data_ptr(), w.data_ptr(), out.data_ptr(),
                              fptr, fbytes, _stream(), ctypes.byref(ms))
    if rc:
        raise SconvError(rc, "sconv_tune")
    return float(ms.value), sconv_plan_name(desc, pooled)
