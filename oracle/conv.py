"""ctypes front end of ``conv_oracle.c`` -- the seven-loop fp64 convolution oracle.

TEST INFRASTRUCTURE ONLY (see the header of ``conv_oracle.c``).  ``build()`` compiles the
C file with gcc into ``oracle/_conv_oracle.so``; nothing here touches the GPU or the HIP
library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "_conv_oracle.so")
_lib = None

SHAPE_FIELDS = ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w",
                "dil_h", "dil_w")


class Shape(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in SHAPE_FIELDS]


def build(force=False):
    """Compile the oracle (gcc -O2 -fopenmp).  Idempotent unless ``force``."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_conv_out_shape.restype = ctypes.c_int
        lib.oracle_conv_out_shape.argtypes = [ctypes.POINTER(Shape),
                                              ctypes.POINTER(ctypes.c_int64),
                                              ctypes.POINTER(ctypes.c_int64)]
        lib.oracle_conv2d_fwd.restype = ctypes.c_int
        lib.oracle_conv2d_fwd.argtypes = [ctypes.POINTER(Shape), ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_int]
        lib.oracle_conv2d_sampled.restype = ctypes.c_int
        lib.oracle_conv2d_sampled.argtypes = [ctypes.POINTER(Shape), ctypes.c_void_p,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                              ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def make_shape(n, c, h, w, k, r, s, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    return Shape(n, c, h, w, k, r, s, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])


def shape_from_layer(layer):
    """``layer`` is a mapping with the 13 SHAPE_FIELDS keys (what the workload module emits)."""
    return Shape(*[int(layer[f]) for f in SHAPE_FIELDS])


def out_shape(shape):
    """(P, Q) by the floor rule, or ``None`` when the descriptor is illegal."""
    p, q = ctypes.c_int64(), ctypes.c_int64()
    rc = _load().oracle_conv_out_shape(ctypes.byref(shape), ctypes.byref(p), ctypes.byref(q))
    return (p.value, q.value) if rc == 0 else None


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def conv2d(shape, x, w, threads=0):
    """Full-tensor oracle.  Returns ``(y64, dnorm, threads_used)``; y64, dnorm are float64
    arrays of shape [N][K][P][Q]."""
    pq = out_shape(shape)
    if pq is None:
        raise ValueError("illegal convolution shape")
    x, w = _f32(x), _f32(w)
    assert x.size == shape.n * shape.c * shape.h * shape.w, "x size does not match the shape"
    assert w.size == shape.k * shape.c * shape.r * shape.s, "w size does not match the shape"
    y = np.empty((shape.n, shape.k, pq[0], pq[1]), dtype=np.float64)
    d = np.empty_like(y)
    used = _load().oracle_conv2d_fwd(ctypes.byref(shape), x.ctypes.data, w.ctypes.data,
                                     y.ctypes.data, None, d.ctypes.data, int(threads))
    if used < 0:
        raise ValueError("oracle rejected the call")
    return y, d, used


def conv2d_sampled(shape, x, w, flat_idx):
    """Oracle value and normaliser of the outputs at flat offsets ``flat_idx`` into NKPQ."""
    x, w = _f32(x), _f32(w)
    assert x.size == shape.n * shape.c * shape.h * shape.w
    assert w.size == shape.k * shape.c * shape.r * shape.s
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    y = np.empty(idx.shape, dtype=np.float64)
    d = np.empty(idx.shape, dtype=np.float64)
    rc = _load().oracle_conv2d_sampled(ctypes.byref(shape), x.ctypes.data, w.ctypes.data,
                                       idx.ctypes.data, idx.size, y.ctypes.data, d.ctypes.data)
    if rc != 0:
        raise ValueError("oracle rejected the call (rc=%d)" % rc)
    return y, d


LAYOUTS = ("NCHW", "NHWC")


def conv2d_layout(shape, x, w, x_layout="NCHW", y_layout="NCHW", threads=0):
    """The same operator on activations stored channels-last (Section 2.1, data layout
    transformation: the values are those of the definition, only their place in memory changes).

    ``x`` is [N][C][H][W] or [N][H][W][C] as ``x_layout`` says, the result (value and normaliser)
    [N][K][P][Q] or [N][P][Q][K] as ``y_layout`` says; weights stay [K][C][R][S].  A layout is a
    permutation of indices, so the oracle permutes, runs the seven loops, and permutes back."""
    assert x_layout in LAYOUTS and y_layout in LAYOUTS
    x = np.asarray(x, dtype=np.float32)
    if x_layout == "NHWC":
        x = x.reshape(shape.n, shape.h, shape.w, shape.c).transpose(0, 3, 1, 2)
    y, d, _ = conv2d(shape, np.ascontiguousarray(x), w, threads=threads)
    if y_layout == "NHWC":
        y, d = (np.ascontiguousarray(t.transpose(0, 2, 3, 1)) for t in (y, d))
    return y, d


def conv2d_fused(shape, x, w, bias=None, residual=None, relu=False, threads=0,
                 x_layout="NCHW", y_layout="NCHW"):
    """The fused operator of Section 2.1 (operator fusion: the sub-graph convolution -> per-channel
    bias -> element-wise addition of a second tensor -> rectifier computed as one operator), written
    out as its definition on top of the seven-loop convolution:

        z[n][k][p][q] = conv(x, w)[n][k][p][q] + bias[k] + residual[n][k][p][q]
        y = max(z, 0) if relu else z

    all in fp64; absent terms are zero.  ``x`` is stored as ``x_layout`` says; the result and the
    residual are stored as ``y_layout`` says ([N][K][P][Q] or channels-last [N][P][Q][K]), so the
    bias runs along axis 1 or along the last axis.  Returns ``(y64, dnorm)`` where dnorm adds |bias|
    and |residual| to the convolution's normaliser: the sum of the magnitudes of everything added
    into an output, which bounds the rounding error of any summation order (the rectifier does
    not increase a difference)."""
    y, d = conv2d_layout(shape, x, w, x_layout, y_layout, threads=threads)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).astype(np.float64)
        assert b.shape == (shape.k,), "bias has one entry per output channel"
        along = (1, shape.k, 1, 1) if y_layout == "NCHW" else (1, 1, 1, shape.k)
        y = y + b.reshape(along)
        d = d + np.abs(b).reshape(along)
    if residual is not None:
        r = np.asarray(residual, dtype=np.float32).astype(np.float64).reshape(y.shape)
        y = y + r
        d = d + np.abs(r)
    if relu:
        y = np.where(y > 0.0, y, 0.0)
    return y, d
