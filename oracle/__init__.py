"""TEST INFRASTRUCTURE -- numpy front end of the plain CPU oracle (oracle/owt_oracle.c).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares nothing with the HIP library and never imports it.

All arrays are C-contiguous numpy arrays, float32 or float64 (the dtype of the
first argument selects the f32 or f64 build of the same loop nests).
Activations are NHWC, filters KRSC, fully-connected weights [O_local, I].
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "owt_oracle.c"), os.path.join(_HERE, "owt_oracle_impl.inc")]
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain C + OpenMP).  Returns the .so path."""
    stale = (not os.path.exists(_LIB_PATH)) or any(
        os.path.getmtime(s) > os.path.getmtime(_LIB_PATH) for s in _SRC)
    if force or stale:
        tmp = _LIB_PATH + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O3", "-march=native", "-fopenmp", "-shared", "-fPIC",
                               "-std=c11", _SRC[0], "-o", tmp, "-lm"])
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _sfx(a):
    if a.dtype == np.float32:
        return "f32", ctypes.c_float
    if a.dtype == np.float64:
        return "f64", ctypes.c_double
    raise TypeError("oracle takes float32 or float64 arrays, got %s" % a.dtype)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _pair(v):
    return (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))


def out_hw(H, W, R, S, stride, pad):
    (sh, sw), (ph, pw) = _pair(stride), _pair(pad)
    return (H + 2 * ph - R) // sh + 1, (W + 2 * pw - S) // sw + 1


def _geom(N, C, H, W, K, R, S, stride, pad):
    (sh, sw), (ph, pw) = _pair(stride), _pair(pad)
    return [ctypes.c_int(v) for v in (N, C, H, W, K, R, S, sh, sw, ph, pw)]


def conv_fwd(x, w, bias=None, stride=1, pad=0, relu=False):
    sfx, _ = _sfx(x)
    x = _c(x, x.dtype); w = _c(w, x.dtype); bias = _c(bias, x.dtype)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    P, Q = out_hw(H, W, R, S, stride, pad)
    y = np.empty((N, P, Q, K), dtype=x.dtype)
    getattr(lib(), "oracle_conv_fwd_" + sfx)(_p(x), _p(w), _p(bias), _p(y),
                                             *_geom(N, C, H, W, K, R, S, stride, pad),
                                             ctypes.c_int(1 if relu else 0))
    return y


def conv_bwd_data(dy, w, hw, stride=1, pad=0, y=None):
    sfx, _ = _sfx(dy)
    dy = _c(dy, dy.dtype); w = _c(w, dy.dtype); y = _c(y, dy.dtype)
    H, W = hw
    K, R, S, C = w.shape
    N, P, Q, K2 = dy.shape
    assert K == K2 and (P, Q) == out_hw(H, W, R, S, stride, pad)
    dx = np.empty((N, H, W, C), dtype=dy.dtype)
    getattr(lib(), "oracle_conv_bwd_data_" + sfx)(_p(dy), _p(y), _p(w), _p(dx),
                                                  *_geom(N, C, H, W, K, R, S, stride, pad))
    return dx


def conv_bwd_filter(x, dy, rs, stride=1, pad=0, y=None, alpha=1.0, beta=0.0,
                    dw=None, db=None, want_db=True):
    """Returns (dw, db).  With beta != 0 pass the old dw (and db); they are updated in a copy."""
    sfx, _ = _sfx(x)
    x = _c(x, x.dtype); dy = _c(dy, x.dtype); y = _c(y, x.dtype)
    R, S = rs
    N, H, W, C = x.shape
    K = dy.shape[3]
    assert dy.shape[:3] == (N,) + out_hw(H, W, R, S, stride, pad)
    dw = np.empty((K, R, S, C), dtype=x.dtype) if dw is None else np.array(dw, dtype=x.dtype, order="C")
    if want_db:
        db = np.empty((K,), dtype=x.dtype) if db is None else np.array(db, dtype=x.dtype, order="C")
    else:
        db = None
    getattr(lib(), "oracle_conv_bwd_filter_" + sfx)(_p(x), _p(dy), _p(y),
                                                    ctypes.c_double(alpha), ctypes.c_double(beta),
                                                    _p(dw), _p(db),
                                                    *_geom(N, C, H, W, K, R, S, stride, pad))
    return dw, db


def conv_bwd_filter_at(x, dy, idx, rs, stride=1, pad=0, y=None):
    """dw[k,r,s,c] for each row (k,r,s,c) of idx, alpha=1, beta=0."""
    sfx, _ = _sfx(x)
    x = _c(x, x.dtype); dy = _c(dy, x.dtype); y = _c(y, x.dtype)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    R, S = rs
    N, H, W, C = x.shape
    K = dy.shape[3]
    out = np.empty((idx.shape[0],), dtype=x.dtype)
    getattr(lib(), "oracle_conv_bwd_filter_at_" + sfx)(_p(x), _p(dy), _p(y), _p(idx),
                                                       ctypes.c_int(idx.shape[0]), _p(out),
                                                       *_geom(N, C, H, W, K, R, S, stride, pad))
    return out


def fc_fwd(x, w, bias=None, relu=False):
    sfx, _ = _sfx(x)
    x = _c(x, x.dtype); w = _c(w, x.dtype); bias = _c(bias, x.dtype)
    N, I = x.shape
    O, I2 = w.shape
    assert I == I2
    y = np.empty((N, O), dtype=x.dtype)
    getattr(lib(), "oracle_fc_fwd_" + sfx)(_p(x), _p(w), _p(bias), _p(y), ctypes.c_int(N),
                                           ctypes.c_int(I), ctypes.c_int(O),
                                           ctypes.c_int(1 if relu else 0))
    return y


def fc_bwd(x, w, dy, y=None, alpha=1.0, beta=0.0, dw=None, db=None, want_dx=True, want_db=True):
    """Returns (dx_partial or None, dw, db or None)."""
    sfx, _ = _sfx(x)
    x = _c(x, x.dtype); w = _c(w, x.dtype); dy = _c(dy, x.dtype); y = _c(y, x.dtype)
    N, I = x.shape
    O = w.shape[0]
    dx = np.empty((N, I), dtype=x.dtype) if want_dx else None
    dw = np.empty((O, I), dtype=x.dtype) if dw is None else np.array(dw, dtype=x.dtype, order="C")
    if want_db:
        db = np.empty((O,), dtype=x.dtype) if db is None else np.array(db, dtype=x.dtype, order="C")
    else:
        db = None
    getattr(lib(), "oracle_fc_bwd_" + sfx)(_p(x), _p(w), _p(y), _p(dy), ctypes.c_double(alpha),
                                           ctypes.c_double(beta), _p(dx), _p(dw), _p(db),
                                           ctypes.c_int(N), ctypes.c_int(I), ctypes.c_int(O))
    return dx, dw, db


def maxpool_fwd(x, win=3, stride=2):
    sfx, _ = _sfx(x)
    x = _c(x, x.dtype)
    N, H, W, C = x.shape
    P, Q = (H - win) // stride + 1, (W - win) // stride + 1
    y = np.empty((N, P, Q, C), dtype=x.dtype)
    am = np.empty((N, P, Q, C), dtype=np.uint8)
    getattr(lib(), "oracle_maxpool_fwd_" + sfx)(_p(x), _p(y), _p(am), *[ctypes.c_int(v) for v in
                                                (N, H, W, C, win, stride)])
    return y, am


def maxpool_bwd(dy, argmax, hw, win=3, stride=2):
    sfx, _ = _sfx(dy)
    dy = _c(dy, dy.dtype)
    argmax = np.ascontiguousarray(argmax, dtype=np.uint8)
    H, W = hw
    N, P, Q, C = dy.shape
    dx = np.empty((N, H, W, C), dtype=dy.dtype)
    getattr(lib(), "oracle_maxpool_bwd_" + sfx)(_p(dy), _p(argmax), _p(dx), *[ctypes.c_int(v) for v in
                                                (N, H, W, C, win, stride)])
    return dx


def sgd_momentum(w, vel, g, mu, eps, omega, gscale=1.0):
    """Section 5 update rule; returns the new (w, vel), inputs untouched."""
    sfx, _ = _sfx(w)
    w2, v2 = np.array(w, dtype=w.dtype, order="C"), np.array(vel, dtype=w.dtype, order="C")
    g = _c(g, w.dtype)
    assert w2.shape == v2.shape == g.shape
    getattr(lib(), "oracle_sgd_momentum_" + sfx)(_p(w2), _p(v2), _p(g), ctypes.c_size_t(w2.size), ctypes.c_double(mu),
                                                 ctypes.c_double(eps), ctypes.c_double(omega), ctypes.c_double(gscale))
    return w2, v2


def logistic_xent(z, labels, col0=0, scale=1.0):
    """Independent logistic units + cross-entropy on this shard's columns: (loss[N], dz[N, O])."""
    sfx, _ = _sfx(z)
    z = _c(z, z.dtype)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    N, O = z.shape
    assert labels.shape == (N,)
    loss, dz = np.empty((N,), dtype=z.dtype), np.empty((N, O), dtype=z.dtype)
    getattr(lib(), "oracle_logistic_xent_" + sfx)(_p(z), _p(labels), _p(loss), _p(dz), ctypes.c_int(N), ctypes.c_int(O),
                                                  ctypes.c_int(col0), ctypes.c_double(scale))
    return loss, dz


def scale_hyperparameters(k, eps, omega):
    """(eps', omega') for a batch k times larger (Section 5)."""
    e2, o2 = ctypes.c_double(), ctypes.c_double()
    lib().oracle_scale_hyperparameters(ctypes.c_double(k), ctypes.c_double(eps), ctypes.c_double(omega),
                                       ctypes.byref(e2), ctypes.byref(o2))
    return e2.value, o2.value


def round_bf16(a):
    """fp32 -> nearest-even bf16 -> fp32 (values stay float32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty_like(a)
    lib().oracle_round_bf16(_p(a), _p(out), ctypes.c_size_t(a.size))
    return out


def num_threads():
    return int(lib().oracle_num_threads())
