"""Python face of the CPU oracle (oracle/cnn_oracle.cpp).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
CPU-baseline leg load this; the GPU library and its binding never do.

Each function forwards numpy arrays to the C++ definition of the same name
(Section 3 of arXiv 1912.05234: conv, mconv, sigmoid, avgpool, backweights,
backbias, backin, backavgpool, forward).  float32 arrays go to the instance
that stores float and sums in double; float64 arrays to the all-double
instance.  Arrays of rank < 4 are given leading unit axes, which does not
change their memory image.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cnn_oracle.cpp")
_LIB = os.path.join(_HERE, "libcnn_oracle.so")

NPARAM = 3898
PARAM_SHAPES = (("k1", (6, 5, 5)), ("b1", (6,)), ("k2", (12, 6, 5, 5)), ("b2", (12,)),
                ("fc", (10, 12, 1, 4, 4)), ("b", (10,)))


def build(force=False):
    """Compile the oracle with the host compiler (no GPU code involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for suf, ct in (("f32", ctypes.c_float), ("f64", ctypes.c_double)):
            getattr(_lib, "oracle_backbias_" + suf).restype = ct
            getattr(_lib, "oracle_grad_image_" + suf).restype = ctypes.c_double
            getattr(_lib, "oracle_train_batch_" + suf).restype = ctypes.c_double
    return _lib


def _suf(a):
    if a.dtype == np.float32:
        return "f32"
    if a.dtype == np.float64:
        return "f64"
    raise TypeError("oracle takes float32 or float64 arrays, got %s" % a.dtype)


def _c(a, dtype=None):
    return np.ascontiguousarray(a, dtype=dtype)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _shape4(shape):
    if len(shape) > 4:
        raise ValueError("rank > 4 not supported")
    s = (1,) * (4 - len(shape)) + tuple(int(x) for x in shape)
    return (ctypes.c_int * 4)(*s), s


def _fn(name, a):
    return getattr(_load(), "oracle_%s_%s" % (name, _suf(a)))


def conv(I, k):
    I, k = _c(I), _c(k, I.dtype)
    if I.ndim != k.ndim:
        raise ValueError("conv needs arrays of equal rank")
    si, _ = _shape4(I.shape)
    sk, _ = _shape4(k.shape)
    out = np.empty(tuple(a - b + 1 for a, b in zip(I.shape, k.shape)), I.dtype)
    _fn("conv", I)(_p(I), si, _p(k), sk, _p(out))
    return out


def mconv(I, k, b):
    I, k, b = _c(I), _c(k, I.dtype), _c(b, I.dtype)
    n = b.shape[0]
    if k.shape[0] != n or k.ndim != I.ndim + 1:
        raise ValueError("mconv: k must be [n, *kernel] with one kernel per bias")
    si, _ = _shape4(I.shape)
    sk, _ = _shape4(k.shape[1:])
    out = np.empty((n,) + tuple(a - c + 1 for a, c in zip(I.shape, k.shape[1:])), I.dtype)
    _fn("mconv", I)(_p(I), si, _p(k), ctypes.c_int(n), sk, _p(b), _p(out))
    return out


def round_bf16(x):
    """Nearest bfloat16 value of every element (ties to even), as float32."""
    x = _c(x, np.float32)
    out = np.empty_like(x)
    _load().oracle_round_bf16(_p(x), ctypes.c_long(x.size), _p(out))
    return out


def sigmoid(x):
    x = _c(x)
    out = np.empty_like(x)
    _fn("sigmoid", x)(_p(x), ctypes.c_long(x.size), _p(out))
    return out


def sigmoid_back(y, d_out):
    y, d_out = _c(y), _c(d_out, y.dtype)
    out = np.empty_like(y)
    _fn("sigmoid_back", y)(_p(y), _p(d_out), ctypes.c_long(y.size), _p(out))
    return out


def avgpool(x):
    x = _c(x)
    H, W = x.shape[-2:]
    lead = int(np.prod(x.shape[:-2], dtype=np.int64))
    out = np.empty(x.shape[:-2] + (H // 2, W // 2), x.dtype)
    _fn("avgpool", x)(_p(x), ctypes.c_long(lead), ctypes.c_int(H), ctypes.c_int(W), _p(out))
    return out


def backavgpool(d_out):
    d_out = _c(d_out)
    Ho, Wo = d_out.shape[-2:]
    lead = int(np.prod(d_out.shape[:-2], dtype=np.int64))
    out = np.empty(d_out.shape[:-2] + (2 * Ho, 2 * Wo), d_out.dtype)
    _fn("backavgpool", d_out)(_p(d_out), ctypes.c_long(lead), ctypes.c_int(Ho), ctypes.c_int(Wo),
                              _p(out))
    return out


def backweights(d_out, inp):
    d_out, inp = _c(d_out), _c(inp, d_out.dtype)
    sd, _ = _shape4(d_out.shape)
    si, _ = _shape4(inp.shape)
    out = np.empty(tuple(a - b + 1 for a, b in zip(inp.shape, d_out.shape)), inp.dtype)
    _fn("backweights", d_out)(_p(d_out), sd, _p(inp), si, _p(out))
    return out


def backbias(d_out):
    d_out = _c(d_out)
    return d_out.dtype.type(_fn("backbias", d_out)(_p(d_out), ctypes.c_long(d_out.size)))


def backin(d_out, k, in_shape):
    d_out, k = _c(d_out), _c(k, d_out.dtype)
    sd, _ = _shape4(d_out.shape)
    sk, _ = _shape4(k.shape)
    si, _ = _shape4(in_shape)
    out = np.empty(tuple(in_shape), d_out.dtype)
    _fn("backin", d_out)(_p(d_out), sd, _p(k), sk, si, _p(out))
    return out


def pack(params, dtype=np.float32):
    """dict or sequence (k1,b1,k2,b2,fc,b) -> one flat [3898] vector."""
    if isinstance(params, dict):
        params = [params[n] for n, _ in PARAM_SHAPES]
    flat = np.concatenate([np.asarray(p, dtype=dtype).ravel() for p in params])
    assert flat.size == NPARAM
    return np.ascontiguousarray(flat)


def unpack(w):
    out, off = {}, 0
    for name, shp in PARAM_SHAPES:
        n = int(np.prod(shp))
        out[name] = w[off:off + n].reshape(shp)
        off += n
    return out


def forward(I, w):
    """One image [28,28], flat weights [3898] -> dict of c1,s1,c2,s2,y."""
    I = _c(I)
    w = _c(w, I.dtype)
    a = {"c1": np.empty((6, 24, 24), I.dtype), "s1": np.empty((6, 12, 12), I.dtype),
         "c2": np.empty((12, 8, 8), I.dtype), "s2": np.empty((12, 4, 4), I.dtype),
         "y": np.empty((10,), I.dtype)}
    _fn("forward", I)(_p(I), _p(w), _p(a["c1"]), _p(a["s1"]), _p(a["c2"]), _p(a["s2"]), _p(a["y"]))
    return a


def grad_image(I, label, w):
    """Loss of one image and its gradient [3898] (float64) w.r.t. the weights."""
    I = _c(I)
    w = _c(w, I.dtype)
    g = np.zeros(NPARAM, np.float64)
    loss = _fn("grad_image", I)(_p(I), ctypes.c_int(int(label)), _p(w), _p(g))
    return loss, g


def train_batch(images, labels, rate, w, want_grad=False):
    """One SGD step in place on w; returns the summed loss (and the summed gradient)."""
    images = _c(images)
    labels = _c(labels, np.int32)
    assert w.dtype == images.dtype and w.flags.c_contiguous and w.size == NPARAM
    B = images.shape[0]
    g = np.zeros(NPARAM, np.float64) if want_grad else None
    loss = _fn("train_batch", images)(_p(images), _p(labels), ctypes.c_int(B), ctypes.c_double(rate),
                                      _p(w), _p(g) if want_grad else None)
    return (loss, g) if want_grad else loss


def evaluate(images, labels, w, want_yhat=True):
    """Forward-only pass over N images -> (yhat [N,10] or None, n_correct, loss_sum)."""
    images = _c(images)
    w = _c(w, images.dtype)
    N = images.shape[0]
    yhat = np.empty((N, 10), images.dtype) if want_yhat else None
    nc = ctypes.c_int64(0)
    ls = ctypes.c_double(0.0)
    lab = _c(labels, np.int32) if labels is not None else None
    _fn("evaluate", images)(_p(images), _p(lab) if lab is not None else None, ctypes.c_long(N), _p(w),
                            _p(yhat) if want_yhat else None, ctypes.byref(nc), ctypes.byref(ls))
    return yhat, nc.value, ls.value
