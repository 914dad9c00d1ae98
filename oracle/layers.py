"""ctypes access to the oracle's C layer functions (oracle/layers.c).

Test infrastructure only.  Arrays are numpy, C-contiguous, logical NC(D)HW, dtype
float32 (liboracle_f32) or float64 (liboracle_f64)."""
import ctypes as C

import numpy as np

from . import build as _build

_libs = {}


def lib(dtype):
    dtype = np.dtype(dtype)
    if dtype not in _libs:
        _build.build(force=False)
        L = C.CDLL(_build.lib_path("float" if dtype == np.float32 else "double"))
        L.orc_softmax_ce.restype = C.c_double
        assert L.orc_real_bytes() == dtype.itemsize
        _libs[dtype] = L
    return _libs[dtype]


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _i(*v):
    return [C.c_int64(int(x)) for x in v]


def _geom(x, k, stride, pad):
    """NC(D)HW array + 2-d or 3-d kernel geometry -> (N,C,D,H,W), k3, s3, p3"""
    nsp = len(k)
    N, Cn = x.shape[:2]
    sp = x.shape[2:]
    assert len(sp) == nsp
    if nsp == 2:
        return (N, Cn, 1) + tuple(sp), (1,) + tuple(k), (1,) + tuple(stride), (0,) + tuple(pad)
    return (N, Cn) + tuple(sp), tuple(k), tuple(stride), tuple(pad)


def _osp(sp, k, s, p):
    return tuple((sp[d] + 2 * p[d] - k[d]) // s[d] + 1 for d in range(len(k)))


def conv_fwd(x, w, stride, pad):
    k = w.shape[2:]
    y = np.empty((x.shape[0], w.shape[0]) + _osp(x.shape[2:], k, stride, pad), x.dtype)
    d5, k3, s3, p3 = _geom(x, k, stride, pad)
    lib(x.dtype).orc_conv_fwd(_p(x), _p(w), _p(y), *_i(*d5, w.shape[0], *k3, *s3, *p3))
    return y


def conv_dgrad(dy, w, xshape, stride, pad):
    k = w.shape[2:]
    dx = np.empty(xshape, dy.dtype)
    d5, k3, s3, p3 = _geom(dx, k, stride, pad)
    lib(dy.dtype).orc_conv_dgrad(_p(dy), _p(w), _p(dx), *_i(*d5, w.shape[0], *k3, *s3, *p3))
    return dx


def conv_wgrad(dy, x, wshape, stride, pad):
    k = wshape[2:]
    dw = np.empty(wshape, x.dtype)
    d5, k3, s3, p3 = _geom(x, k, stride, pad)
    lib(x.dtype).orc_conv_wgrad(_p(dy), _p(x), _p(dw), *_i(*d5, wshape[0], *k3, *s3, *p3))
    return dw


def bn_fwd(x, gamma, beta, eps):
    N, Cn = x.shape[:2]
    S = int(np.prod(x.shape[2:]))
    y = np.empty_like(x)
    mean = np.empty(Cn, x.dtype)
    istd = np.empty(Cn, x.dtype)
    lib(x.dtype).orc_bn_fwd(_p(x), _p(gamma), _p(beta), _p(y), _p(mean), _p(istd),
                            *_i(N, Cn, S), C.c_double(eps))
    return y, mean, istd


def bn_bwd(x, dy, gamma, mean, istd):
    N, Cn = x.shape[:2]
    S = int(np.prod(x.shape[2:]))
    dx = np.empty_like(x)
    dg = np.empty(Cn, x.dtype)
    db = np.empty(Cn, x.dtype)
    lib(x.dtype).orc_bn_bwd(_p(x), _p(dy), _p(gamma), _p(mean), _p(istd), _p(dx), _p(dg), _p(db),
                            *_i(N, Cn, S))
    return dx, dg, db


def relu_fwd(x):
    y = np.empty_like(x)
    lib(x.dtype).orc_relu_fwd(_p(x), _p(y), *_i(x.size))
    return y


def relu_bwd(y, dy):
    dx = np.empty_like(y)
    lib(y.dtype).orc_relu_bwd(_p(y), _p(dy), _p(dx), *_i(y.size))
    return dx


def maxpool_fwd(x, k, stride, pad):
    y = np.empty(x.shape[:2] + _osp(x.shape[2:], k, stride, pad), x.dtype)
    d5, k3, s3, p3 = _geom(x, k, stride, pad)
    lib(x.dtype).orc_maxpool_fwd(_p(x), _p(y), *_i(d5[0] * d5[1], *d5[2:], *k3, *s3, *p3))
    return y


def maxpool_bwd(x, dy, k, stride, pad):
    dx = np.empty_like(x)
    d5, k3, s3, p3 = _geom(x, k, stride, pad)
    lib(x.dtype).orc_maxpool_bwd(_p(x), _p(dy), _p(dx), *_i(d5[0] * d5[1], *d5[2:], *k3, *s3, *p3))
    return dx


def gavgpool_fwd(x):
    y = np.empty(x.shape[:2], x.dtype)
    lib(x.dtype).orc_gavgpool_fwd(_p(x), _p(y), *_i(x.shape[0] * x.shape[1], int(np.prod(x.shape[2:]))))
    return y


def gavgpool_bwd(dy, xshape):
    dx = np.empty(xshape, dy.dtype)
    lib(dy.dtype).orc_gavgpool_bwd(_p(dy), _p(dx), *_i(xshape[0] * xshape[1], int(np.prod(xshape[2:]))))
    return dx


def fc_fwd(x, w, b):
    x2 = np.ascontiguousarray(x.reshape(x.shape[0], -1))
    y = np.empty((x2.shape[0], w.shape[0]), x.dtype)
    lib(x.dtype).orc_fc_fwd(_p(x2), _p(w), _p(b), _p(y), *_i(x2.shape[0], x2.shape[1], w.shape[0]))
    return y


def fc_bwd(x, w, dy):
    x2 = np.ascontiguousarray(x.reshape(x.shape[0], -1))
    dx = np.empty_like(x2)
    dw = np.empty_like(w)
    db = np.empty(w.shape[0], x.dtype)
    lib(x.dtype).orc_fc_bwd(_p(x2), _p(w), _p(dy), _p(dx), _p(dw), _p(db),
                            *_i(x2.shape[0], x2.shape[1], w.shape[0]))
    return dx.reshape(x.shape), dw, db


def softmax_ce(z, t):
    dz = np.empty_like(z)
    t = np.ascontiguousarray(t, np.int32)
    loss = lib(z.dtype).orc_softmax_ce(_p(z), _p(t), _p(dz), *_i(*z.shape))
    return float(loss), dz
