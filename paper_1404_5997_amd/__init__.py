"""ctypes binding of libowt (include/owt.h): argument marshalling only.

Every function has the name and argument order of its C entry point.  Tensor
arguments are torch tensors living on the GPU (torch is used for device memory
and streams only); the binding passes their data pointers and the current
stream through.  A non-OK status raises OwtError carrying owt_last_error().

There is no CPU fallback: if libowt.so has not been built, importing this
package raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libowt.so")

OWT_OK, OWT_EINVAL, OWT_EUNSUPPORTED, OWT_EWORKSPACE, OWT_ELAUNCH = 0, 1, 2, 3, 4
OWT_F32, OWT_BF16 = 0, 1
OWT_BIAS, OWT_RELU = 1, 2
OWT_PASS_FWD, OWT_PASS_BWD_DATA, OWT_PASS_BWD_FILTER = 0, 1, 2
OWT_FORCE_NO_DIRECT, OWT_FORCE_ONLY_DIRECT, OWT_FORCE_NO_BF16_MFMA = 1, 2, 4
OWT_FORCE_FC_ONE_LAUNCH, OWT_FORCE_FC_TWO_LAUNCHES = 8, 16

EXPORTS = (
    "owt_conv_workspace_bytes", "owt_fc_workspace_bytes", "owt_conv_fwd", "owt_conv_bwd_data",
    "owt_conv_bwd_filter", "owt_fc_shard_fwd", "owt_fc_shard_bwd", "owt_maxpool_fwd",
    "owt_maxpool_bwd", "owt_last_error", "owt_abi_version", "owt_selftest_host", "owt_conv_plan_describe", "owt_conv_autotune",
    "owt_conv_bwd_data_relu_in", "owt_maxpool_bwd_relu", "owt_sgd_momentum_update", "owt_scale_hyperparameters",
    "owt_logistic_xent", "owt_fc_autotune", "owt_test_force_variant",
    "owt_conv_bwd_filter_static", "owt_static_scratch_bytes",
)


class OwtError(RuntimeError):
    def __init__(self, status, message):
        RuntimeError.__init__(self, "owt status %d: %s" % (status, message))
        self.status = status


class owt_conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dtype")] + \
               [("flags", ctypes.c_uint)]


class owt_fc_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("N", "I", "O_total", "workers", "rank", "dtype")] + \
               [("flags", ctypes.c_uint)]


if not os.path.exists(LIB_PATH):
    raise ImportError("libowt.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(hipcc, gfx950).  There is no fallback path.")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _sz, _f, _i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_int
_cd, _fd = ctypes.POINTER(owt_conv_desc), ctypes.POINTER(owt_fc_desc)
_lib.owt_conv_workspace_bytes.restype = _sz
_lib.owt_conv_workspace_bytes.argtypes = [_cd, _i]
_lib.owt_fc_workspace_bytes.restype = _sz
_lib.owt_fc_workspace_bytes.argtypes = [_fd, _i]
_lib.owt_conv_fwd.argtypes = [_cd, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.owt_conv_bwd_data.argtypes = [_cd, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.owt_conv_bwd_data_relu_in.argtypes = [_cd, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.owt_maxpool_bwd_relu.argtypes = [_i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp]
_lib.owt_conv_bwd_filter.argtypes = [_cd, _vp, _vp, _vp, _f, _f, _vp, _vp, _vp, _sz, _vp]
_lib.owt_conv_bwd_filter_static.argtypes = [_cd, _vp, _vp, _vp, _f, _f, _vp, _vp, _vp]
_lib.owt_static_scratch_bytes.restype = _sz
_lib.owt_conv_autotune.argtypes = [_cd, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.owt_fc_autotune.argtypes = [_fd, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.owt_fc_shard_fwd.argtypes = [_fd, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.owt_fc_shard_bwd.argtypes = [_fd, _vp, _vp, _vp, _vp, _f, _f, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.owt_maxpool_fwd.argtypes = [_i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]
_lib.owt_maxpool_bwd.argtypes = [_i, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]
_d = ctypes.c_double
_lib.owt_sgd_momentum_update.argtypes = [_sz, _vp, _vp, _vp, _f, _f, _f, _f, _vp, _vp]
_lib.owt_scale_hyperparameters.argtypes = [_d, _d, _d, ctypes.POINTER(_d), ctypes.POINTER(_d)]
_lib.owt_logistic_xent.argtypes = [_i, _i, _i, _i, _vp, _vp, _f, _vp, _vp, _vp]
_lib.owt_last_error.restype = ctypes.c_char_p
_lib.owt_abi_version.restype = _i
_lib.owt_conv_plan_describe.argtypes = [_cd, _i, ctypes.c_char_p, _sz]
_lib.owt_test_force_variant.argtypes = [_i, _i, ctypes.c_uint]
_lib.owt_test_force_variant.restype = None


def _ptr(t):
    """Device pointer of a torch tensor (or a raw int / None passed through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("owt takes dense row-major tensors")
    return t.data_ptr()


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(status):
    if status != OWT_OK:
        raise OwtError(status, owt_last_error())


def owt_last_error():
    return _lib.owt_last_error().decode()


def owt_abi_version():
    return _lib.owt_abi_version()


def owt_conv_plan_describe(desc, pass_):
    buf = ctypes.create_string_buffer(256)
    n = _lib.owt_conv_plan_describe(ctypes.byref(desc), pass_, buf, ctypes.c_size_t(256))
    if n < 0:
        raise OwtError(OWT_EINVAL, owt_last_error())
    return buf.value.decode()


def owt_test_force_variant(tile=-1, splitk=0, flags=0):
    _lib.owt_test_force_variant(tile, splitk, flags)


def owt_selftest_host():
    return _lib.owt_selftest_host()


def conv_desc(N, C, H, W, K, R, S, stride=1, pad=0, dtype=OWT_F32, flags=0):
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return owt_conv_desc(N, C, H, W, K, R, S, sh, sw, ph, pw, dtype, flags)


def fc_desc(N, I, O_total, workers, rank=0, dtype=OWT_F32, flags=0):
    return owt_fc_desc(N, I, O_total, workers, rank, dtype, flags)


def owt_conv_workspace_bytes(desc, pass_):
    n = _lib.owt_conv_workspace_bytes(ctypes.byref(desc), pass_)
    if n == ctypes.c_size_t(-1).value:
        raise OwtError(OWT_EINVAL, owt_last_error())
    return n


def owt_fc_workspace_bytes(desc, pass_):
    n = _lib.owt_fc_workspace_bytes(ctypes.byref(desc), pass_)
    if n == ctypes.c_size_t(-1).value:
        raise OwtError(OWT_EINVAL, owt_last_error())
    return n


def owt_conv_fwd(desc, x, w, bias, y, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_conv_fwd(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), p, n, _stream(stream)))


def owt_conv_bwd_data(desc, dy, y_or_null, w, dx, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_conv_bwd_data(ctypes.byref(desc), _ptr(dy), _ptr(y_or_null), _ptr(w), _ptr(dx), p, n,
                                  _stream(stream)))


def owt_conv_bwd_data_relu_in(desc, dy, y_or_null, w, x, dx, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_conv_bwd_data_relu_in(ctypes.byref(desc), _ptr(dy), _ptr(y_or_null), _ptr(w), _ptr(x), _ptr(dx),
                                          p, n, _stream(stream)))


def owt_conv_bwd_filter(desc, x, dy, y_or_null, alpha, beta, dw, dbias_or_null, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_conv_bwd_filter(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(y_or_null), alpha, beta,
                                    _ptr(dw), _ptr(dbias_or_null), p, n, _stream(stream)))


def owt_conv_bwd_filter_static(desc, x, dy, y_or_null, alpha, beta, dw, dbias_or_null, stream=None):
    _check(_lib.owt_conv_bwd_filter_static(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(y_or_null), alpha, beta,
                                           _ptr(dw), _ptr(dbias_or_null), _stream(stream)))


def owt_static_scratch_bytes():
    return _lib.owt_static_scratch_bytes()


def owt_conv_autotune(desc, pass_, x, w, bias, y, dy, dx, dw, dbias_or_null, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_conv_autotune(ctypes.byref(desc), pass_, _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(dy), _ptr(dx),
                                  _ptr(dw), _ptr(dbias_or_null), p, n, _stream(stream)))


def owt_fc_shard_fwd(desc, x, w, bias, y, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_fc_shard_fwd(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), p, n, _stream(stream)))


def owt_fc_autotune(desc, x, w, bias, y, dy, dx_partial, dw, dbias_or_null, ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_fc_autotune(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(dy), _ptr(dx_partial),
                                _ptr(dw), _ptr(dbias_or_null), p, n, _stream(stream)))


def owt_fc_shard_bwd(desc, x, w, y_or_null, dy, alpha, beta, dx_partial_or_null, dw, dbias_or_null,
                     ws=None, stream=None):
    p, n = _ws(ws)
    _check(_lib.owt_fc_shard_bwd(ctypes.byref(desc), _ptr(x), _ptr(w), _ptr(y_or_null), _ptr(dy), alpha, beta,
                                 _ptr(dx_partial_or_null), _ptr(dw), _ptr(dbias_or_null), p, n, _stream(stream)))


def owt_maxpool_fwd(N, H, W, C, win, stride, dtype, x, y, argmax, stream=None):
    _check(_lib.owt_maxpool_fwd(N, H, W, C, win, stride, dtype, _ptr(x), _ptr(y), _ptr(argmax), _stream(stream)))


def owt_maxpool_bwd(N, H, W, C, win, stride, dtype, dy, argmax, dx, stream=None):
    _check(_lib.owt_maxpool_bwd(N, H, W, C, win, stride, dtype, _ptr(dy), _ptr(argmax), _ptr(dx), _stream(stream)))


def owt_sgd_momentum_update(n, w, vel, g, mu, eps, omega, gscale=1.0, w_bf16=None, stream=None):
    _check(_lib.owt_sgd_momentum_update(n, _ptr(w), _ptr(vel), _ptr(g), mu, eps, omega, gscale, _ptr(w_bf16),
                                        _stream(stream)))


def owt_scale_hyperparameters(k, eps, omega):
    e2, o2 = _d(), _d()
    _check(_lib.owt_scale_hyperparameters(k, eps, omega, ctypes.byref(e2), ctypes.byref(o2)))
    return e2.value, o2.value


def owt_logistic_xent(N, O_local, col_offset, dtype, z, labels, scale, loss, dz, stream=None):
    _check(_lib.owt_logistic_xent(N, O_local, col_offset, dtype, _ptr(z), _ptr(labels), scale, _ptr(loss), _ptr(dz),
                                  _stream(stream)))


def owt_maxpool_bwd_relu(N, H, W, C, win, stride, dtype, dy, argmax, y_pooled, dx, stream=None):
    _check(_lib.owt_maxpool_bwd_relu(N, H, W, C, win, stride, dtype, _ptr(dy), _ptr(argmax), _ptr(y_pooled), _ptr(dx),
                                     _stream(stream)))
