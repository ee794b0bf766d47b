"""ctypes front end of the CPU oracle (``sconv_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the benchmark's
CPU-baseline leg.  The GPU package never imports this, and this never imports the GPU package.
Everything here is argument marshalling plus two closed-form counters (Eq. 1, Eq. 2 and the
multiply/add counts of Section 5.4); the arithmetic of the method lives in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sconv_oracle.c")
_LIB = os.path.join(_HERE, "libsconv_oracle.so")

FMT_ECR = 0
FMT_PECR = 1


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride", "pad", "groups",
                 "pool_h", "pool_w", "pool_stride")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2; OpenMP over (n, k) in oracle_conv and over the rows in oracle_spmv)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.POINTER
        f32, i32, i64, f64 = ctypes.c_float, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        lib.oracle_output_dims.argtypes = [P(Shape), P(i32), P(i32), P(i32), P(i32)]
        lib.oracle_output_dims.restype = None
        lib.oracle_eq3_n_o.argtypes = [f64] * 5
        lib.oracle_eq3_n_o.restype = f64
        lib.oracle_encode_sizes.argtypes = [P(Shape), ctypes.c_int, P(i64), P(i64)]
        lib.oracle_encode_sizes.restype = None
        lib.oracle_encode.argtypes = [P(Shape), ctypes.c_int, P(f32), P(f32), P(i32), P(i32)]
        lib.oracle_encode.restype = None
        lib.oracle_spmv.argtypes = [P(Shape), i64, P(f32), P(i32), P(i32), P(f32), P(f64)]
        lib.oracle_spmv.restype = None
        lib.oracle_conv.argtypes = [P(Shape), P(f32), P(f32), ctypes.c_int, P(f64), P(f64)]
        lib.oracle_conv.restype = None
        lib.oracle_conv_at.argtypes = [P(Shape), P(f32), P(f32), ctypes.c_int, i64, P(i32), P(f64), P(f64)]
        lib.oracle_conv_at.restype = None
        lib.oracle_maxpool.argtypes = [P(Shape), P(f64), P(f64), P(f64), P(f64)]
        lib.oracle_maxpool.restype = None
        lib.oracle_conv_pool.argtypes = [P(Shape), P(f32), P(f32), P(f64), P(f64), P(f64), P(f64)]
        lib.oracle_conv_pool.restype = None
        lib.oracle_add_bias.argtypes = [i32, i32, i64, P(f32), ctypes.c_int, P(f64), P(f64)]
        lib.oracle_add_bias.restype = None
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_set_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _f32(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs are fp32")
    return a


def make_shape(x_shape, w_shape, stride=1, pad=0, groups=1, pool=None) -> Shape:
    N, C, H, W = x_shape
    K, Cg, R, S = w_shape
    if Cg * groups != C:
        raise ValueError("filter channel count does not match C / groups")
    ph, pw, ps = pool if pool is not None else (0, 0, 0)
    return Shape(N, C, H, W, K, R, S, stride, pad, groups, ph, pw, ps)


def output_dims(shape: Shape) -> Tuple[int, int, int, int]:
    lib = _load()
    v = [ctypes.c_int32() for _ in range(4)]
    lib.oracle_output_dims(ctypes.byref(shape), *[ctypes.byref(t) for t in v])
    return tuple(t.value for t in v)


def eq3_n_o(I_w, k_w, c_s, p_w, p_s) -> float:
    """Eq. (3) as printed (no flooring)."""
    return _load().oracle_eq3_n_o(I_w, k_w, c_s, p_w, p_s)


def encode_sizes(shape: Shape, fmt: int) -> Tuple[int, int]:
    lib = _load()
    rows, L = ctypes.c_int64(), ctypes.c_int64()
    lib.oracle_encode_sizes(ctypes.byref(shape), fmt, ctypes.byref(rows), ctypes.byref(L))
    return rows.value, L.value


def encode(x: np.ndarray, w_shape, fmt: int, stride=1, pad=0, groups=1, pool=None):
    """Algorithm 1 (fmt=FMT_ECR) / Algorithm 3 (fmt=FMT_PECR): (values[rows,L], index[rows,L], count[rows])."""
    lib = _load()
    x = _f32(x)
    shape = make_shape(x.shape, w_shape, stride, pad, groups, pool)
    rows, L = encode_sizes(shape, fmt)
    values = np.empty((rows, L), np.float32)
    index = np.empty((rows, L), np.int32)
    count = np.empty((rows,), np.int32)
    lib.oracle_encode(ctypes.byref(shape), fmt, _ptr(x, ctypes.c_float), _ptr(values, ctypes.c_float),
                      _ptr(index, ctypes.c_int32), _ptr(count, ctypes.c_int32))
    return values, index, count


def spmv(values, index, count, w, x_shape, stride=1, pad=0, groups=1, pool=None) -> np.ndarray:
    """Algorithm 2 on an encoding: out[rows, K/groups] in fp64."""
    lib = _load()
    w = _f32(w)
    shape = make_shape(x_shape, w.shape, stride, pad, groups, pool)
    rows = values.shape[0]
    out = np.empty((rows, shape.K // shape.groups), np.float64)
    lib.oracle_spmv(ctypes.byref(shape), rows, _ptr(np.ascontiguousarray(values), ctypes.c_float),
                    _ptr(np.ascontiguousarray(index), ctypes.c_int32),
                    _ptr(np.ascontiguousarray(count), ctypes.c_int32),
                    _ptr(w, ctypes.c_float), _ptr(out, ctypes.c_double))
    return out


def conv(x, w, stride=1, pad=0, groups=1, relu=False, want_absdot=True):
    """Plain fp64 convolution: (y[N,K,OH,OW], absdot or None)."""
    lib = _load()
    x, w = _f32(x), _f32(w)
    shape = make_shape(x.shape, w.shape, stride, pad, groups)
    OH, OW, _, _ = output_dims(shape)
    y = np.empty((shape.N, shape.K, OH, OW), np.float64)
    a = np.empty_like(y) if want_absdot else None
    lib.oracle_conv(ctypes.byref(shape), _ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                    1 if relu else 0, _ptr(y, ctypes.c_double), _ptr(a, ctypes.c_double))
    return y, a


def conv_bias(x, w, bias, stride=1, pad=0, groups=1, relu=False):
    """Convolution layer with bias: the plain fp64 sums, + bias[k], then the optional ReLU:
    (y[N,K,OH,OW], absdot including |bias|)."""
    lib = _load()
    y, a = conv(x, w, stride, pad, groups, relu=False)
    b = _f32(bias)
    N, K, OH, OW = y.shape
    if b.shape != (K,):
        raise ValueError("bias must have one value per filter")
    lib.oracle_add_bias(N, K, OH * OW, _ptr(b, ctypes.c_float), 1 if relu else 0,
                        _ptr(y, ctypes.c_double), _ptr(a, ctypes.c_double))
    return y, a


def conv_pool_bias(x, w, bias, pool, stride=1, pad=0, groups=1):
    """Fused definition with bias: conv, + bias[k], ReLU, max pooling: (z[N,K,PH,PW], scale)."""
    y, a = conv_bias(x, w, bias, stride, pad, groups, relu=True)
    return maxpool(y, pool, a)


def conv_at(x, w, points, stride=1, pad=0, groups=1, relu=False):
    """The plain fp64 convolution at listed outputs: points[i] = (n, k, oh, ow) -> (y[i], absdot[i])."""
    lib = _load()
    x, w = _f32(x), _f32(w)
    shape = make_shape(x.shape, w.shape, stride, pad, groups)
    pts = np.ascontiguousarray(points, np.int32).reshape(-1, 4)
    y = np.empty((pts.shape[0],), np.float64)
    a = np.empty_like(y)
    lib.oracle_conv_at(ctypes.byref(shape), _ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                       1 if relu else 0, pts.shape[0], _ptr(pts, ctypes.c_int32),
                       _ptr(y, ctypes.c_double), _ptr(a, ctypes.c_double))
    return y, a


def maxpool(y: np.ndarray, pool, scale: Optional[np.ndarray] = None):
    """Max pooling of an fp64 [N,K,OH,OW] tensor with window (p_h, p_w, p_s)."""
    lib = _load()
    y = np.ascontiguousarray(y, np.float64)
    N, K, OH, OW = y.shape
    # only N, K, the pooling fields and an (H, R, pad, stride) set that reproduces OH/OW matter
    shape = Shape(N, 1, OH, OW, K, 1, 1, 1, 0, 1, pool[0], pool[1], pool[2])
    _, _, PH, PW = output_dims(shape)
    z = np.empty((N, K, PH, PW), np.float64)
    so = np.empty_like(z) if scale is not None else None
    si = np.ascontiguousarray(scale, np.float64) if scale is not None else None
    lib.oracle_maxpool(ctypes.byref(shape), _ptr(y, ctypes.c_double), _ptr(si, ctypes.c_double),
                       _ptr(z, ctypes.c_double), _ptr(so, ctypes.c_double))
    return z, so


def conv_pool(x, w, pool, stride=1, pad=0, groups=1):
    """Fused definition: conv, ReLU, max pooling: (z[N,K,PH,PW], scale)."""
    lib = _load()
    x, w = _f32(x), _f32(w)
    shape = make_shape(x.shape, w.shape, stride, pad, groups, pool)
    OH, OW, PH, PW = output_dims(shape)
    tmp = np.empty((shape.N, shape.K, OH, OW), np.float64)
    atmp = np.empty_like(tmp)
    z = np.empty((shape.N, shape.K, PH, PW), np.float64)
    sc = np.empty_like(z)
    lib.oracle_conv_pool(ctypes.byref(shape), _ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                         _ptr(tmp, ctypes.c_double), _ptr(atmp, ctypes.c_double),
                         _ptr(z, ctypes.c_double), _ptr(sc, ctypes.c_double))
    return z, sc


# ---- closed-form counters -------------------------------------------------------------------

def dense_op_counts(i_w, i_h, k_w, k_h, c_s) -> Tuple[int, int]:
    """Eq. (1) and Eq. (2): multiplications and additions of one dense single-channel convolution."""
    windows = ((i_w - k_w) // c_s + 1) * ((i_h - k_h) // c_s + 1)
    return windows * (k_w * k_h), windows * (k_w * k_h - 1)


def sparse_op_counts(count: np.ndarray) -> Tuple[int, int]:
    """Section 5.4: one multiplication per stored nonzero, one addition fewer per non-empty window."""
    c = np.maximum(np.asarray(count, np.int64), 0)
    return int(c.sum()), int(np.maximum(c - 1, 0).sum())


class one_thread:
    """Context manager: the OpenMP loop of oracle_conv runs on one thread inside (timing aid)."""

    def __enter__(self):
        self.before = _load().oracle_set_threads(1)
        return self

    def __exit__(self, *exc):
        _load().oracle_set_threads(self.before)
        return False


def threads():
    """Threads the OpenMP loop of oracle_conv uses."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return int(v.split(",")[0])
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))
