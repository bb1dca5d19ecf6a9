"""ctypes/numpy binding of the CPU oracle (test infrastructure only).

`Oracle("float")` drives libcgo_f32.so, `Oracle("double")` libcgo_f64.so; both
are built from the same C sources by oracle/build.py.  Arrays go in and come
out as C-contiguous numpy arrays of the matching dtype.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("N", "C", "H", "W", "M", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w", "groups")]


def conv_desc(N, Cin, H, W, M, k, stride=1, pad=0, groups=1, kw=None):
    return ConvDesc(N, Cin, H, W, M, k, k if kw is None else kw, stride, stride, pad, pad, groups)


class Oracle:
    def __init__(self, real="float"):
        assert real in ("float", "double")
        path = _build.lib_path(real)
        if not os.path.exists(path):
            _build.build(force=False)
        self.lib = C.CDLL(path)
        self.dtype = np.float32 if real == "float" else np.float64
        self.creal = C.c_float if real == "float" else C.c_double
        self.lib.cgo_maxpool_out.restype = C.c_int
        self.lib.cgo_num_threads.restype = C.c_int

    # -- helpers -----------------------------------------------------------------
    def _a(self, a):
        a = np.ascontiguousarray(a, dtype=self.dtype)
        return a

    @staticmethod
    def _p(a):
        return a.ctypes.data_as(C.c_void_p)

    def num_threads(self):
        return int(self.lib.cgo_num_threads())

    def set_num_threads(self, n):
        self.lib.cgo_set_num_threads(C.c_int(n))

    # -- convolution ---------------------------------------------------------------
    def conv_out_shape(self, d):
        oh, ow = C.c_int(), C.c_int()
        rc = self.lib.cgo_conv_out_shape(C.byref(d), C.byref(oh), C.byref(ow))
        if rc:
            raise ValueError("invalid convolution descriptor")
        return oh.value, ow.value

    def conv_fwd(self, d, x, w, bias=None):
        x, w = self._a(x), self._a(w)
        OH, OW = self.conv_out_shape(d)
        y = np.empty((d.N, d.M, OH, OW), self.dtype)
        b = self._a(bias) if bias is not None else None
        rc = self.lib.cgo_conv_fwd(C.byref(d), self._p(x), self._p(w),
                                   self._p(b) if b is not None else None, self._p(y))
        assert rc == 0
        return y

    def conv_bwd_data(self, d, dy, w):
        dy, w = self._a(dy), self._a(w)
        dx = np.empty((d.N, d.C, d.H, d.W), self.dtype)
        rc = self.lib.cgo_conv_bwd_data(C.byref(d), self._p(dy), self._p(w), self._p(dx))
        assert rc == 0
        return dx

    def conv_bwd_weight(self, d, x, dy, want_bias=True):
        x, dy = self._a(x), self._a(dy)
        dw = np.empty((d.M, d.C // d.groups, d.KH, d.KW), self.dtype)
        db = np.empty(d.M, self.dtype) if want_bias else None
        rc = self.lib.cgo_conv_bwd_weight(C.byref(d), self._p(x), self._p(dy), self._p(dw),
                                          self._p(db) if want_bias else None)
        assert rc == 0
        return dw, db

    # -- elementwise / pooling -----------------------------------------------------
    def relu_fwd(self, x):
        x = self._a(x)
        y = np.empty_like(x)
        self.lib.cgo_relu_fwd(C.c_size_t(x.size), self._p(x), self._p(y))
        return y

    def relu_bwd(self, x, dy):
        x, dy = self._a(x), self._a(dy)
        dx = np.empty_like(x)
        self.lib.cgo_relu_bwd(C.c_size_t(x.size), self._p(x), self._p(dy), self._p(dx))
        return dx

    def maxpool_out(self, H, k, s, p):
        return int(self.lib.cgo_maxpool_out(H, k, s, p))

    def maxpool_fwd(self, x, k, s, p):
        x = self._a(x)
        N, Ch, H, W = x.shape
        OH, OW = self.maxpool_out(H, k, s, p), self.maxpool_out(W, k, s, p)
        y = np.empty((N, Ch, OH, OW), self.dtype)
        am = np.empty((N, Ch, OH, OW), np.int32)
        self.lib.cgo_maxpool_fwd(N, Ch, H, W, k, s, p, self._p(x), self._p(y), self._p(am))
        return y, am

    def maxpool_bwd(self, xshape, k, s, p, dy, argmax):
        dy = self._a(dy)
        N, Ch, H, W = xshape
        dx = np.empty(xshape, self.dtype)
        am = np.ascontiguousarray(argmax, np.int32)
        self.lib.cgo_maxpool_bwd(N, Ch, H, W, k, s, p, self._p(dy), self._p(am), self._p(dx))
        return dx

    def lrn_fwd(self, x, size, alpha, beta, kappa):
        x = self._a(x)
        N, Ch, H, W = x.shape
        y, sc = np.empty_like(x), np.empty_like(x)
        self.lib.cgo_lrn_fwd(N, Ch, H * W, size, C.c_double(alpha), C.c_double(beta), C.c_double(kappa),
                             self._p(x), self._p(y), self._p(sc))
        return y, sc

    def lrn_bwd(self, x, y, scale, dy, size, alpha, beta):
        x, y, scale, dy = map(self._a, (x, y, scale, dy))
        N, Ch, H, W = x.shape
        dx = np.empty_like(x)
        self.lib.cgo_lrn_bwd(N, Ch, H * W, size, C.c_double(alpha), C.c_double(beta),
                             self._p(x), self._p(y), self._p(scale), self._p(dy), self._p(dx))
        return dx

    def avgpool_fwd(self, x):
        x = self._a(x)
        N, Ch, H, W = x.shape
        y = np.empty((N, Ch, 1, 1), self.dtype)
        self.lib.cgo_avgpool_fwd(N, Ch, H * W, self._p(x), self._p(y))
        return y

    def avgpool_bwd(self, xshape, dy):
        dy = self._a(dy)
        N, Ch, H, W = xshape
        dx = np.empty(xshape, self.dtype)
        self.lib.cgo_avgpool_bwd(N, Ch, H * W, self._p(dy), self._p(dx))
        return dx

    # -- fully connected -------------------------------------------------------------
    def fc_fwd(self, x, W, bias=None):
        x, W = self._a(x), self._a(W)
        B, IN = x.shape
        OUT = W.shape[0]
        y = np.empty((B, OUT), self.dtype)
        b = self._a(bias) if bias is not None else None
        self.lib.cgo_fc_fwd(B, IN, OUT, self._p(x), self._p(W), self._p(b) if b is not None else None,
                            self._p(y))
        return y

    def fc_bwd_data(self, dy, W):
        dy, W = self._a(dy), self._a(W)
        B, OUT = dy.shape
        IN = W.shape[1]
        dx = np.empty((B, IN), self.dtype)
        self.lib.cgo_fc_bwd_data(B, IN, OUT, self._p(dy), self._p(W), self._p(dx))
        return dx

    def fc_bwd_weight(self, x, dy):
        x, dy = self._a(x), self._a(dy)
        B, IN = x.shape
        OUT = dy.shape[1]
        dW, db = np.empty((OUT, IN), self.dtype), np.empty(OUT, self.dtype)
        self.lib.cgo_fc_bwd_weight(B, IN, OUT, self._p(x), self._p(dy), self._p(dW), self._p(db))
        return dW, db

    def dropout(self, x, mask, p):
        x = self._a(x)
        m = np.ascontiguousarray(mask, np.uint8)
        assert m.size == x.size
        y = np.empty_like(x)
        self.lib.cgo_dropout(C.c_size_t(x.size), C.c_double(p), m.ctypes.data_as(C.c_void_p),
                             self._p(x), self._p(y))
        return y

    def softmax_ce(self, z, labels):
        z = self._a(z)
        B, Cn = z.shape
        lab = np.ascontiguousarray(labels, np.int32)
        loss = np.zeros(1, self.dtype)
        dz = np.empty_like(z)
        self.lib.cgo_softmax_ce(B, Cn, self._p(z), lab.ctypes.data_as(C.c_void_p), self._p(loss), self._p(dz))
        return loss[0], dz

    # -- Eq. 1 + solver history ----------------------------------------------------------
    def grad_reduce_sgd(self, w, v, g_local, g_peers, lr, mu, wd, grad_scale=1.0, order="sequential"):
        """In place on w and v (which must be contiguous arrays of the oracle's dtype).
        order: "sequential" (local, then peers left to right) or "tree" (binomial reduction tree)."""
        assert w.dtype == self.dtype and v.dtype == self.dtype and w.flags.c_contiguous and v.flags.c_contiguous
        g_local = self._a(g_local)
        peers = [self._a(p) for p in g_peers]
        n = w.size
        assert v.size == n and g_local.size == n and all(p.size == n for p in peers)
        arr = (C.c_void_p * max(len(peers), 1))(*[p.ctypes.data for p in peers])
        r = self.creal
        fn = {"sequential": self.lib.cgo_grad_reduce_sgd, "tree": self.lib.cgo_grad_reduce_sgd_tree}[order]
        fn(self._p(w), self._p(v), self._p(g_local), arr, C.c_int(len(peers)),
                                     C.c_size_t(n), r(lr), r(mu), r(wd), r(grad_scale))
