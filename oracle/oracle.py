"""ctypes access to liboracle.so (oracle.cpp): argument marshalling only.

TEST INFRASTRUCTURE: see the header of oracle.cpp.  Arrays are NCHW / OIHW numpy
arrays of float32 ("f32": float storage, double accumulation) or float64 ("f64").
"""
import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

__all__ = [
    "build", "lib", "conv_fwd", "conv_dgrad", "conv_wgrad", "bn_fwd", "bn_bwd", "relu_fwd",
    "relu_bwd", "maxpool_fwd", "maxpool_bwd", "gap_fwd", "gap_bwd", "fc_fwd", "fc_bwd",
    "softmax_ce", "train_step", "out_dim", "BN_EPS",
]

BN_EPS = 1e-5


def build(force: bool = False) -> str:
    """Compile oracle.cpp with g++ (-O3 -march=native -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared",
                               "-std=c++17", "-Wall", "-o", _LIB, _SRC])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for sfx in ("f32", "f64"):
            getattr(_lib, f"oracle_softmax_ce_{sfx}").restype = C.c_double
            getattr(_lib, f"oracle_train_step_{sfx}").restype = C.c_int
    return _lib


def out_dim(size: int, r: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - r) // stride + 1


def _sfx(a: np.ndarray) -> str:
    if a.dtype == np.float32:
        return "f32"
    if a.dtype == np.float64:
        return "f64"
    raise TypeError(f"oracle takes float32 or float64, got {a.dtype}")


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a: np.ndarray, like: Optional[np.ndarray] = None) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if like is not None and a.dtype != like.dtype:
        raise TypeError("mixed dtypes")
    return a


def conv_fwd(x, w, stride=1, pad=0):
    x = _c(x); w = _c(w, x)
    n, cin, h, wd = x.shape
    cout, cin2, r, s = w.shape
    assert cin == cin2
    y = np.zeros((n, cout, out_dim(h, r, stride, pad), out_dim(wd, s, stride, pad)), x.dtype)
    getattr(lib(), f"oracle_conv_fwd_{_sfx(x)}")(_p(x), _p(w), _p(y), n, cin, h, wd, cout, r, s, stride, pad)
    return y


def conv_dgrad(dy, w, x_shape, stride=1, pad=0):
    dy = _c(dy); w = _c(w, dy)
    n, cin, h, wd = x_shape
    cout, _, r, s = w.shape
    assert dy.shape == (n, cout, out_dim(h, r, stride, pad), out_dim(wd, s, stride, pad))
    dx = np.zeros(x_shape, dy.dtype)
    getattr(lib(), f"oracle_conv_dgrad_{_sfx(dy)}")(_p(dy), _p(w), _p(dx), n, cin, h, wd, cout, r, s, stride, pad)
    return dx


def conv_wgrad(x, dy, w_shape, stride=1, pad=0):
    x = _c(x); dy = _c(dy, x)
    n, cin, h, wd = x.shape
    cout, _, r, s = w_shape
    assert dy.shape == (n, cout, out_dim(h, r, stride, pad), out_dim(wd, s, stride, pad))
    dw = np.zeros(w_shape, x.dtype)
    getattr(lib(), f"oracle_conv_wgrad_{_sfx(x)}")(_p(x), _p(dy), _p(dw), n, cin, h, wd, cout, r, s, stride, pad)
    return dw


def bn_fwd(x, gamma, beta, eps=BN_EPS):
    """-> (y, mean float64[C], istd float64[C])"""
    x = _c(x); gamma = _c(gamma, x); beta = _c(beta, x)
    n, c = x.shape[:2]
    hw = int(np.prod(x.shape[2:]))
    y = np.zeros_like(x)
    mean = np.zeros(c, np.float64); istd = np.zeros(c, np.float64)
    getattr(lib(), f"oracle_bn_fwd_{_sfx(x)}")(_p(x), _p(gamma), _p(beta), _p(y), _p(mean), _p(istd),
                                                n, c, hw, C.c_double(eps))
    return y, mean, istd


def bn_bwd(x, dy, gamma, mean, istd):
    """-> (dx, dgamma, dbeta)"""
    x = _c(x); dy = _c(dy, x); gamma = _c(gamma, x)
    mean = np.ascontiguousarray(mean, np.float64); istd = np.ascontiguousarray(istd, np.float64)
    n, c = x.shape[:2]
    hw = int(np.prod(x.shape[2:]))
    dx = np.zeros_like(x); dg = np.zeros(c, x.dtype); db = np.zeros(c, x.dtype)
    getattr(lib(), f"oracle_bn_bwd_{_sfx(x)}")(_p(x), _p(dy), _p(gamma), _p(mean), _p(istd), _p(dx),
                                                _p(dg), _p(db), n, c, hw)
    return dx, dg, db


def relu_fwd(x):
    x = _c(x); y = np.zeros_like(x)
    getattr(lib(), f"oracle_relu_fwd_{_sfx(x)}")(_p(x), _p(y), C.c_size_t(x.size))
    return y


def relu_bwd(y, dy):
    y = _c(y); dy = _c(dy, y); dx = np.zeros_like(y)
    getattr(lib(), f"oracle_relu_bwd_{_sfx(y)}")(_p(y), _p(dy), _p(dx), C.c_size_t(y.size))
    return dx


def maxpool_fwd(x, r=3, stride=2, pad=1):
    """-> (y, arg int32: flat iy*W+ix of the winner inside each (n,c) plane)"""
    x = _c(x)
    n, c, h, wd = x.shape
    ho, wo = out_dim(h, r, stride, pad), out_dim(wd, r, stride, pad)
    y = np.zeros((n, c, ho, wo), x.dtype); arg = np.zeros((n, c, ho, wo), np.int32)
    getattr(lib(), f"oracle_maxpool_fwd_{_sfx(x)}")(_p(x), _p(y), _p(arg), n, c, h, wd, r, r, stride, pad)
    return y, arg


def maxpool_bwd(dy, arg, x_shape):
    dy = _c(dy); arg = np.ascontiguousarray(arg, np.int32)
    n, c, h, wd = x_shape
    dx = np.zeros(x_shape, dy.dtype)
    getattr(lib(), f"oracle_maxpool_bwd_{_sfx(dy)}")(_p(dy), _p(arg), _p(dx), n, c, h, wd, dy.shape[2], dy.shape[3])
    return dx


def gap_fwd(x):
    x = _c(x)
    n, c = x.shape[:2]
    y = np.zeros((n, c), x.dtype)
    getattr(lib(), f"oracle_gap_fwd_{_sfx(x)}")(_p(x), _p(y), n, c, int(np.prod(x.shape[2:])))
    return y


def gap_bwd(dy, x_shape):
    dy = _c(dy)
    n, c = x_shape[:2]
    dx = np.zeros(x_shape, dy.dtype)
    getattr(lib(), f"oracle_gap_bwd_{_sfx(dy)}")(_p(dy), _p(dx), n, c, int(np.prod(x_shape[2:])))
    return dx


def fc_fwd(x, param, cout):
    """param = [W (cout x cin, row major) | b (cout)]"""
    x = _c(x); param = _c(param, x)
    n, cin = x.shape
    assert param.size == cout * cin + cout
    y = np.zeros((n, cout), x.dtype)
    getattr(lib(), f"oracle_fc_fwd_{_sfx(x)}")(_p(x), _p(param), _p(y), n, cin, cout)
    return y


def fc_bwd(x, param, dy):
    """-> (dx, dparam)"""
    x = _c(x); param = _c(param, x); dy = _c(dy, x)
    n, cin = x.shape
    cout = dy.shape[1]
    dx = np.zeros_like(x); dparam = np.zeros_like(param)
    getattr(lib(), f"oracle_fc_bwd_{_sfx(x)}")(_p(x), _p(param), _p(dy), _p(dx), _p(dparam), n, cin, cout)
    return dx, dparam


def softmax_ce(z, labels):
    """-> (loss float, dz)"""
    z = _c(z); labels = np.ascontiguousarray(labels, np.int32)
    n, classes = z.shape
    dz = np.zeros_like(z)
    loss = getattr(lib(), f"oracle_softmax_ce_{_sfx(z)}")(_p(z), _p(labels), _p(dz), n, classes)
    return float(loss), dz


def train_step(spec_array: np.ndarray, in_chw: Sequence[int], params: List[np.ndarray],
               images: np.ndarray, labels: np.ndarray, lr: float, eps: float = BN_EPS,
               want_acts: Optional[Sequence[int]] = None, act_sizes: Optional[dict] = None):
    """One forward / backward / SGD step.

    spec_array: int32 [n_layers, 9] layer records; params: one array per layer
    (conv OIHW, bn [gamma|beta], fc [W|b]), all float32 or all float64, NOT
    modified.  Returns (loss, new_params, grads[, acts]) where acts maps layer id
    -> flat forward output for the ids in want_acts (sizes given by act_sizes)."""
    recs = np.ascontiguousarray(spec_array, np.int32)
    nl = recs.shape[0]
    images = _c(images)
    dt = images.dtype
    sfx = _sfx(images)
    labels = np.ascontiguousarray(labels, np.int32)
    newp = [np.array(p, dtype=dt, copy=True).ravel() for p in params]
    grads = [np.zeros(p.size, dt) for p in newp]
    acts = {}
    if want_acts:
        for i in want_acts:
            acts[i] = np.zeros(act_sizes[i], dt)
    PP = C.c_void_p * nl
    pp = PP(*[p.ctypes.data if p.size else None for p in newp])
    gg = PP(*[g.ctypes.data if g.size else None for g in grads])
    aa = PP(*[acts[i].ctypes.data if i in acts else None for i in range(nl)])
    loss = C.c_double(0.0)
    rc = getattr(lib(), f"oracle_train_step_{sfx}")(
        _p(recs), nl, int(in_chw[0]), int(in_chw[1]), int(in_chw[2]), images.shape[0], pp, gg,
        aa if want_acts else None, _p(images), _p(labels), C.c_double(lr), C.c_double(eps),
        C.byref(loss))
    if rc != 0:
        raise ValueError(f"oracle_train_step: malformed layer record {-rc - 1}")
    if want_acts:
        return loss.value, newp, grads, acts
    return loss.value, newp, grads
