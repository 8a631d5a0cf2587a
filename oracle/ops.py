"""ctypes binding of ``asgd_oracle.c`` (argument marshalling only).

Every array is float64 in canonical layout: activations [N,C,H,W], conv filters
[Cout,Cin,k,k], FC weights [out,in].
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asgd_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_U8 = ctypes.POINTER(ctypes.c_uint8)
_I32 = ctypes.POINTER(ctypes.c_int32)


def build(force=False):
    """Compile the C oracle with gcc (OpenMP over the host cores)."""
    global _lib
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-Wall", "-Wextra", "-shared",
                               "-fPIC", _SRC, "-o", _LIB, "-lm"])
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_softmax_ce.restype = ctypes.c_double
        _lib.oracle_dropout_threshold.restype = ctypes.c_uint32
        _lib.oracle_dropout_threshold.argtypes = [ctypes.c_double]
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _d(a):
    return a.ctypes.data_as(_D)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _extent(n, k, s, p):
    return (n + 2 * p - k) // s + 1


def num_threads():
    return int(_load().oracle_num_threads())


def conv_fwd(x, w, b, stride, pad):
    x, w, b = _f64(x), _f64(w), _f64(b)
    N, Cin, H, W = x.shape
    Cout, Cin2, k, k2 = w.shape
    assert Cin == Cin2 and k == k2 and b.shape == (Cout,)
    y = np.empty((N, Cout, _extent(H, k, stride, pad), _extent(W, k, stride, pad)))
    _load().oracle_conv_fwd(_d(x), _d(w), _d(b), _d(y), N, Cin, H, W, Cout, k, stride, pad)
    return y


def conv_bwd_data(dy, w, in_hw, stride, pad):
    dy, w = _f64(dy), _f64(w)
    N, Cout = dy.shape[:2]
    _, Cin, k, _ = w.shape
    H, W = in_hw
    assert dy.shape == (N, Cout, _extent(H, k, stride, pad), _extent(W, k, stride, pad))
    dx = np.empty((N, Cin, H, W))
    _load().oracle_conv_bwd_data(_d(dy), _d(w), _d(dx), N, Cin, H, W, Cout, k, stride, pad)
    return dx


def conv_bwd_weight(x, dy, k, stride, pad):
    x, dy = _f64(x), _f64(dy)
    N, Cin, H, W = x.shape
    Cout = dy.shape[1]
    assert dy.shape == (N, Cout, _extent(H, k, stride, pad), _extent(W, k, stride, pad))
    dw = np.empty((Cout, Cin, k, k))
    db = np.empty((Cout,))
    _load().oracle_conv_bwd_weight(_d(x), _d(dy), _d(dw), _d(db), N, Cin, H, W, Cout, k, stride, pad)
    return dw, db


def relu_fwd(y):
    y = _f64(y)
    r = np.empty_like(y)
    _load().oracle_relu_fwd(_d(y), _d(r), ctypes.c_size_t(y.size))
    return r


def relu_bwd(y, dr):
    y, dr = _f64(y), _f64(dr)
    assert y.shape == dr.shape
    dy = np.empty_like(y)
    _load().oracle_relu_bwd(_d(y), _d(dr), _d(dy), ctypes.c_size_t(y.size))
    return dy


def maxpool_fwd(r, k, stride):
    r = _f64(r)
    N, C, H, W = r.shape
    Ho, Wo = _extent(H, k, stride, 0), _extent(W, k, stride, 0)
    p = np.empty((N, C, Ho, Wo))
    idx = np.empty((N, C, Ho, Wo), dtype=np.uint8)
    _load().oracle_maxpool_fwd(_d(r), _d(p), idx.ctypes.data_as(_U8), N, C, H, W, k, stride)
    return p, idx


def maxpool_gather(r, idx, k, stride):
    """Values of r at the given window positions (see oracle_maxpool_gather)."""
    r = _f64(r)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    N, C, H, W = r.shape
    assert idx.shape == (N, C, _extent(H, k, stride, 0), _extent(W, k, stride, 0)) and idx.max() < k * k
    p = np.empty(idx.shape)
    _load().oracle_maxpool_gather(_d(r), idx.ctypes.data_as(_U8), _d(p), N, C, H, W, k, stride)
    return p


def maxpool_bwd(dp, idx, in_hw, k, stride):
    dp = _f64(dp)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    N, C = dp.shape[:2]
    H, W = in_hw
    assert dp.shape == idx.shape == (N, C, _extent(H, k, stride, 0), _extent(W, k, stride, 0))
    dr = np.empty((N, C, H, W))
    _load().oracle_maxpool_bwd(_d(dp), idx.ctypes.data_as(_U8), _d(dr), N, C, H, W, k, stride)
    return dr


def lrn_fwd(a, size, alpha, beta, k):
    """Cross-channel local response normalisation of a [N,C,H,W] tensor."""
    a = _f64(a)
    N, C, H, W = a.shape
    b = np.empty_like(a)
    _load().oracle_lrn_fwd(_d(a), _d(b), N, C, H, W, int(size), ctypes.c_double(alpha), ctypes.c_double(beta), ctypes.c_double(k))
    return b


def lrn_bwd(a, db, size, alpha, beta, k):
    a, db = _f64(a), _f64(db)
    N, C, H, W = a.shape
    assert db.shape == a.shape
    da = np.empty_like(a)
    _load().oracle_lrn_bwd(_d(a), _d(db), _d(da), N, C, H, W, int(size), ctypes.c_double(alpha), ctypes.c_double(beta),
                           ctypes.c_double(k))
    return da


def fc_fwd(x, w, b):
    x, w, b = _f64(x), _f64(w), _f64(b)
    N, nin = x.shape
    nout = w.shape[0]
    assert w.shape == (nout, nin) and b.shape == (nout,)
    y = np.empty((N, nout))
    _load().oracle_fc_fwd(_d(x), _d(w), _d(b), _d(y), N, nin, nout)
    return y


def fc_bwd(x, w, dy, need_dx=True):
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    N, nin = x.shape
    nout = w.shape[0]
    assert dy.shape == (N, nout)
    dx = np.empty((N, nin)) if need_dx else None
    dw = np.empty((nout, nin))
    db = np.empty((nout,))
    _load().oracle_fc_bwd(_d(x), _d(w), _d(dy), _d(dx) if need_dx else None, _d(dw), _d(db), N, nin, nout)
    return dx, dw, db


def dropout_threshold(p):
    return int(_load().oracle_dropout_threshold(float(p)))


def dropout_mask(count, seed, step, worker, layer, p):
    mask = np.empty((count,), dtype=np.uint8)
    _load().oracle_dropout_mask(mask.ctypes.data_as(_U8), ctypes.c_size_t(count), ctypes.c_uint64(seed),
                                ctypes.c_uint64(step), ctypes.c_uint32(worker), ctypes.c_uint32(layer),
                                ctypes.c_uint32(dropout_threshold(p)))
    return mask


def dropout_apply(r, mask, scale=1.0):
    r = _f64(r)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    assert mask.size == r.size
    h = np.empty_like(r)
    _load().oracle_dropout_apply(_d(r), mask.ctypes.data_as(_U8), ctypes.c_double(scale), _d(h),
                                 ctypes.c_size_t(r.size))
    return h


def softmax_ce(z, labels, want_grad=True):
    z = _f64(z)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    N, C = z.shape
    assert labels.shape == (N,) and labels.min() >= 0 and labels.max() < C
    dz = np.empty_like(z) if want_grad else None
    loss = _load().oracle_softmax_ce(_d(z), labels.ctypes.data_as(_I32), _d(dz) if want_grad else None, N, C)
    return float(loss), dz


def apply_update(w, v, g, lr, mu, wd):
    """In place on the float64 arrays ``w`` and ``v``."""
    assert w.dtype == v.dtype == np.float64 and w.flags.c_contiguous and v.flags.c_contiguous
    g = _f64(g)
    assert w.size == v.size == g.size
    _load().oracle_apply_update(_d(w), _d(v), _d(g), ctypes.c_size_t(w.size), ctypes.c_double(lr),
                                ctypes.c_double(mu), ctypes.c_double(wd))


def apply_adagrad(w, h, g, lr, eps, wd):
    """In place on the float64 arrays ``w`` (parameters) and ``h`` (sum of squared gradients)."""
    assert w.dtype == h.dtype == np.float64 and w.flags.c_contiguous and h.flags.c_contiguous
    g = _f64(g)
    assert w.size == h.size == g.size
    _load().oracle_apply_adagrad(_d(w), _d(h), _d(g), ctypes.c_size_t(w.size), ctypes.c_double(lr), ctypes.c_double(eps),
                                 ctypes.c_double(wd))


def apply_adadelta(w, a, b, g, rho, eps, wd):
    """In place on the float64 arrays ``w``, ``a`` (running mean of squared gradients), ``b`` (of squared steps)."""
    assert w.dtype == a.dtype == b.dtype == np.float64 and w.flags.c_contiguous and a.flags.c_contiguous and b.flags.c_contiguous
    g = _f64(g)
    assert w.size == a.size == b.size == g.size
    _load().oracle_apply_adadelta(_d(w), _d(a), _d(b), _d(g), ctypes.c_size_t(w.size), ctypes.c_double(rho), ctypes.c_double(eps),
                                  ctypes.c_double(wd))


def snapshot_bf16(params_f32):
    """fp32 array -> uint16 array of bf16 bit patterns (round to nearest even)."""
    p = np.ascontiguousarray(params_f32, dtype=np.float32)
    out = np.empty(p.shape, dtype=np.uint16)
    _load().oracle_snapshot_bf16(p.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                 out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), ctypes.c_size_t(p.size))
    return out


def bf16_to_f64(bits):
    """Widen bf16 bit patterns (uint16) exactly to float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def round_bf16(a):
    """Round a float64 array to bf16-representable values (via fp32, ties to even), in a copy."""
    out = np.array(a, dtype=np.float64, order="C")
    _load().oracle_round_bf16(_d(out), ctypes.c_size_t(out.size))
    return out


def schedule(T, seed, n_workers=4, max_stale=3):
    worker = np.empty((T,), dtype=np.int32)
    read_version = np.empty((T,), dtype=np.int32)
    _load().oracle_schedule(worker.ctypes.data_as(_I32), read_version.ctypes.data_as(_I32), T,
                            ctypes.c_uint64(seed), n_workers, max_stale)
    return worker, read_version
