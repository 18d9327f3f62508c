"""CPU checker (test infrastructure only): numpy-facing wrappers over stanza_oracle.c.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It never imports the GPU package and is never a fallback for it.

`lib("f32")` / `lib("f64")` give the checker compiled with float or double
storage (sums are always accumulated in double).  All arrays are C-contiguous
numpy arrays in the layouts stated at the top of stanza_oracle.c.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_BUILD = os.path.join(_HERE, "_build")
_SRC = os.path.join(_HERE, "stanza_oracle.c")


def build(force: bool = False) -> None:
    """Compile the checker twice (float and double storage) with gcc."""
    os.makedirs(_BUILD, exist_ok=True)
    for tag, real in (("f32", "float"), ("f64", "double")):
        out = os.path.join(_BUILD, f"liboracle_{tag}.so")
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                               f"-DREAL={real}", _SRC, "-o", out, "-lm"])


class _ConvD(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w")]


class _PoolD(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C", "win_h", "win_w", "stride_h", "stride_w",
                                          "pad_h", "pad_w", "relu")]


@dataclass(frozen=True)
class ConvGeom:
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad: int = 0
    pad_w: int = -1             # horizontal padding when it differs from the vertical one (1xn / nx1 filters); -1: same

    @property
    def pw(self):
        return self.pad if self.pad_w < 0 else self.pad_w

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pw - self.S) // self.stride + 1

    def c(self):
        return _ConvD(self.N, self.H, self.W, self.C, self.K, self.R, self.S, self.stride, self.stride, self.pad, self.pw)


@dataclass(frozen=True)
class PoolGeom:
    N: int
    H: int
    W: int
    C: int
    win: int
    stride: int
    pad: int = 0
    relu: bool = True

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.win) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.win) // self.stride + 1

    def c(self):
        return _PoolD(self.N, self.H, self.W, self.C, self.win, self.win, self.stride, self.stride,
                      self.pad, self.pad, int(self.relu))


class Oracle:
    """One compiled flavour of the checker."""

    def __init__(self, tag: str):
        build()
        self.tag = tag
        self.dtype = np.float32 if tag == "f32" else np.float64
        self._l = C.CDLL(os.path.join(_BUILD, f"liboracle_{tag}.so"))
        assert self._l.oracle_real_bytes() == np.dtype(self.dtype).itemsize
        for name in ("oracle_conv_fwd_at", "oracle_conv_bwd_data_at", "oracle_conv_bwd_weight_at",
                     "oracle_colsum_at", "oracle_fc_fwd_at", "oracle_softmax_ce", "oracle_softmax_ce_part"):
            getattr(self._l, name).restype = C.c_double

    def threads(self) -> int:
        return int(self._l.oracle_threads())

    # -- helpers
    def arr(self, a):
        return np.ascontiguousarray(a, dtype=self.dtype)

    def _p(self, a):
        if a is None:
            return None
        assert a.dtype == self.dtype and a.flags.c_contiguous, (a.dtype, a.flags.c_contiguous)
        return a.ctypes.data_as(C.c_void_p)

    # -- convolution
    def conv_fwd(self, g: ConvGeom, x, w, bias=None, relu=False):
        assert x.shape == (g.N, g.H, g.W, g.C) and w.shape == (g.K, g.R, g.S, g.C)
        y = np.empty((g.N, g.Ho, g.Wo, g.K), self.dtype)
        self._l.oracle_conv_fwd(C.byref(g.c()), self._p(x), self._p(w), self._p(bias), int(relu), self._p(y))
        return y

    def conv_fwd_at(self, g, x, w, bias, relu, n, p, q, k):
        return self._l.oracle_conv_fwd_at(C.byref(g.c()), self._p(x), self._p(w), self._p(bias), int(relu),
                                          int(n), int(p), int(q), int(k))

    def conv_bwd_data(self, g: ConvGeom, dy, w):
        assert dy.shape == (g.N, g.Ho, g.Wo, g.K) and w.shape == (g.K, g.R, g.S, g.C)
        dx = np.empty((g.N, g.H, g.W, g.C), self.dtype)
        self._l.oracle_conv_bwd_data(C.byref(g.c()), self._p(dy), self._p(w), self._p(dx))
        return dx

    def conv_bwd_data_at(self, g, dy, w, n, h, ww, c):
        return self._l.oracle_conv_bwd_data_at(C.byref(g.c()), self._p(dy), self._p(w), int(n), int(h), int(ww), int(c))

    def conv_bwd_weight(self, g: ConvGeom, x, dy):
        assert x.shape == (g.N, g.H, g.W, g.C) and dy.shape == (g.N, g.Ho, g.Wo, g.K)
        dw = np.empty((g.K, g.R, g.S, g.C), self.dtype)
        db = np.empty((g.K,), self.dtype)
        self._l.oracle_conv_bwd_weight(C.byref(g.c()), self._p(x), self._p(dy), self._p(dw), self._p(db))
        return dw, db

    def conv_bwd_weight_at(self, g, x, dy, k, r, s, c):
        return self._l.oracle_conv_bwd_weight_at(C.byref(g.c()), self._p(x), self._p(dy), int(k), int(r), int(s), int(c))

    def colsum_at(self, a2d, j):
        rows, cols = a2d.shape
        return self._l.oracle_colsum_at(self._p(a2d), C.c_size_t(rows), C.c_size_t(cols), C.c_size_t(j))

    def relu_bwd(self, dy, y):
        dz = np.empty_like(dy)
        self._l.oracle_relu_bwd(C.c_size_t(dy.size), self._p(dy), self._p(y), self._p(dz))
        return dz

    # -- pooling
    def pool_relu_fwd(self, g: PoolGeom, x):
        assert x.shape == (g.N, g.H, g.W, g.C)
        y = np.empty((g.N, g.Ho, g.Wo, g.C), self.dtype)
        am = np.empty((g.N, g.Ho, g.Wo, g.C), np.uint8)
        self._l.oracle_pool_relu_fwd(C.byref(g.c()), self._p(x), self._p(y), am.ctypes.data_as(C.c_void_p))
        return y, am

    def pool_relu_bwd(self, g: PoolGeom, dy, y, am):
        assert dy.shape == (g.N, g.Ho, g.Wo, g.C) and am.dtype == np.uint8
        dx = np.empty((g.N, g.H, g.W, g.C), self.dtype)
        self._l.oracle_pool_relu_bwd(C.byref(g.c()), self._p(dy), self._p(y), am.ctypes.data_as(C.c_void_p), self._p(dx))
        return dx

    def avgpool_fwd(self, g: PoolGeom, x):
        assert x.shape == (g.N, g.H, g.W, g.C)
        y = np.empty((g.N, g.Ho, g.Wo, g.C), self.dtype)
        self._l.oracle_avgpool_fwd(C.byref(g.c()), self._p(x), self._p(y))
        return y

    def avgpool_bwd(self, g: PoolGeom, dy):
        assert dy.shape == (g.N, g.Ho, g.Wo, g.C)
        dx = np.empty((g.N, g.H, g.W, g.C), self.dtype)
        self._l.oracle_avgpool_bwd(C.byref(g.c()), self._p(dy), self._p(dx))
        return dx

    # -- residual add, global average pool
    def add_relu_fwd(self, a, b):
        o = np.empty_like(a)
        self._l.oracle_add_relu_fwd(C.c_size_t(a.size), self._p(a), self._p(b), self._p(o))
        return o

    def gap_fwd(self, x):
        n, h, w, c = x.shape
        f = np.empty((n, 1, 1, c), self.dtype)
        self._l.oracle_gap_fwd(n, h * w, c, self._p(x), self._p(f))
        return f

    def gap_bwd(self, df, shape):
        n, h, w, c = shape
        dx = np.empty(shape, self.dtype)
        self._l.oracle_gap_bwd(n, h * w, c, self._p(np.ascontiguousarray(df.reshape(n, c))), self._p(dx))
        return dx

    # -- batch normalisation over the rows of an NHWC tensor (training mode)
    def bn_fwd(self, x, gamma, beta, eps=1e-5, relu=False, run_mean=None, run_var=None, mom=0.1):
        """Returns y, mean [C], istd [C]; run_mean / run_var are updated in place when given."""
        c = x.shape[-1]
        rows = x.size // c
        y = np.empty_like(x)
        mean, istd = np.empty(c, self.dtype), np.empty(c, self.dtype)
        self._l.oracle_bn_fwd(C.c_size_t(rows), c, self._p(x), self._p(gamma), self._p(beta), C.c_double(eps), int(relu),
                              self._p(y), self._p(mean), self._p(istd), self._p(run_mean), self._p(run_var), C.c_double(mom))
        return y, mean, istd

    def bn_bwd(self, x, dy, gamma, mean, istd):
        """dy: gradient of the pre-ReLU output.  Returns dx, dgamma, dbeta."""
        c = x.shape[-1]
        rows = x.size // c
        dx = np.empty_like(x)
        dg, db = np.empty(c, self.dtype), np.empty(c, self.dtype)
        self._l.oracle_bn_bwd(C.c_size_t(rows), c, self._p(x), self._p(dy), self._p(gamma), self._p(mean), self._p(istd),
                              self._p(dx), self._p(dg), self._p(db))
        return dx, dg, db

    # -- FC
    def fc_fwd(self, a, w, b=None, relu=False):
        n, cin = a.shape
        out = w.shape[0]
        assert w.shape == (out, cin)
        z = np.empty((n, out), self.dtype)
        self._l.oracle_fc_fwd(n, cin, out, self._p(a), self._p(w), self._p(b), int(relu), self._p(z))
        return z

    def fc_fwd_at(self, a, w, b, i, o, relu=False):
        cin = a.shape[1]
        return self._l.oracle_fc_fwd_at(cin, self._p(a[i]), self._p(w[o]), self._p(b), int(o), int(relu))

    def fc_bwd(self, a, w, dz, need_da=True):
        n, cin = a.shape
        out = w.shape[0]
        dw = np.empty((out, cin), self.dtype)
        db = np.empty((out,), self.dtype)
        da = np.empty((n, cin), self.dtype) if need_da else None
        self._l.oracle_fc_bwd(n, cin, out, self._p(a), self._p(w), self._p(dz), self._p(dw), self._p(db), self._p(da))
        return dw, db, da

    def softmax_ce(self, z, labels):
        n, classes = z.shape
        labels = np.ascontiguousarray(labels, np.int32)
        dz = np.empty_like(z)
        pred = np.empty((n,), np.int32)
        loss = self._l.oracle_softmax_ce(n, classes, self._p(z), labels.ctypes.data_as(C.c_void_p), self._p(dz),
                                         pred.ctypes.data_as(C.c_void_p))
        return loss, dz, pred

    def softmax_ce_part(self, z, labels, n_global):
        """One of several FC workers: its rows' share of the loss and the gradient, both normalised by the global batch."""
        n, classes = z.shape
        labels = np.ascontiguousarray(labels, np.int32)
        dz = np.empty_like(z)
        pred = np.empty((n,), np.int32)
        loss = self._l.oracle_softmax_ce_part(n, int(n_global), classes, self._p(z), labels.ctypes.data_as(C.c_void_p), self._p(dz),
                                              pred.ctypes.data_as(C.c_void_p))
        return loss, dz, pred

    # -- optimiser (in place on w, v)
    def sgd_momentum(self, w, v, g, lr, momentum, wd):
        self._l.oracle_sgd_momentum(C.c_size_t(w.size), self._p(w), self._p(v), self._p(g),
                                    C.c_double(lr), C.c_double(momentum), C.c_double(wd))

    def ps_aggregate(self, w, v, grads, scale, lr, momentum, wd):
        K = len(grads)
        ptrs = (C.c_void_p * K)(*[g.ctypes.data for g in grads])
        for g in grads:
            assert g.dtype == self.dtype and g.flags.c_contiguous and g.size == w.size
        self._l.oracle_ps_aggregate(C.c_size_t(w.size), self._p(w), self._p(v), ptrs, K,
                                    C.c_double(scale), C.c_double(lr), C.c_double(momentum), C.c_double(wd))


_LIBS = {}


def lib(tag: str = "f32") -> Oracle:
    if tag not in _LIBS:
        _LIBS[tag] = Oracle(tag)
    return _LIBS[tag]
