"""Thin ctypes binding of the C ABI in ``include/asgd.h`` (argument marshalling only).

Every function has the name of the C entry point it calls.  Device buffers are
torch tensors on the GPU (PyTorch is used for device memory and streams only);
every step of the computation runs in the library's HIP kernels.  If the
library has not been built, loading it raises: there is no fallback path.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libasgd_mi355x.so")

F32, BF16 = 0, 1
LAYER_CONV, LAYER_RELU, LAYER_MAXPOOL, LAYER_FC, LAYER_DROPOUT, LAYER_SOFTMAX_CE, LAYER_LRN = 1, 2, 3, 4, 5, 6, 7
DEBUG_OUTPUT, DEBUG_ARGMAX, DEBUG_MASK = 0, 1, 2
OK, EINVAL, ESHAPE, ENOMEM, EHIP, EALIGN = 0, -1, -2, -3, -4, -5

EXPORTS = ["asgd_net_create", "asgd_net_prepare", "asgd_net_destroy", "asgd_net_set_serial", "asgd_param_count", "asgd_param_layout",
           "asgd_layer_shape", "asgd_workspace_bytes", "asgd_fwd_bwd", "asgd_fwd_bwd_static", "asgd_static_workspace_bytes",
           "asgd_apply_update", "asgd_snapshot",
           "asgd_apply_update_snapshot", "asgd_train_step", "asgd_train_step_fused",
           "asgd_debug_get", "asgd_profile_begin", "asgd_profile_end", "asgd_schedule_generate", "asgd_replay_run", "asgd_replay_nsync_run", "asgd_accumulate", "asgd_apply_update_adagrad", "asgd_apply_update_adadelta",
           "asgd_last_error"]
KERNEL_CLASSES = ["conv_fwd", "conv_dgrad", "conv_wgrad", "fc_fwd", "fc_dgrad", "fc_wgrad", "pool_fwd", "pool_bwd",
                  "bias_grad", "softmax_ce", "layout", "update", "lrn"]


class LayerDesc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("out", ctypes.c_int32), ("k", ctypes.c_int32), ("stride", ctypes.c_int32),
                ("pad", ctypes.c_int32), ("p", ctypes.c_float), ("scale", ctypes.c_float), ("bias", ctypes.c_float), ("groups", ctypes.c_int32)]


class TensorInfo(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_int32), ("kind", ctypes.c_int32), ("w_offset", ctypes.c_uint64),
                ("w_count", ctypes.c_uint64), ("b_offset", ctypes.c_uint64), ("b_count", ctypes.c_uint64),
                ("w_shape", ctypes.c_int32 * 4)]


class ProfileEntry(ctypes.Structure):
    _fields_ = [("kclass", ctypes.c_int32), ("launches", ctypes.c_int32), ("ms", ctypes.c_double),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]


class AsgdError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("asgd error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: run `python -m paper_1312_6186_amd.build` (there is no fallback path)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
        L.asgd_net_create.argtypes = [ctypes.POINTER(LayerDesc), ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int, ctypes.POINTER(vp)]
        L.asgd_net_prepare.argtypes = [vp]
        L.asgd_net_destroy.argtypes = [vp]
        L.asgd_net_set_serial.argtypes = [vp, ctypes.c_int]
        L.asgd_param_count.argtypes = [vp]
        L.asgd_param_count.restype = ctypes.c_size_t
        L.asgd_param_layout.argtypes = [vp, ctypes.POINTER(TensorInfo), ctypes.c_int]
        L.asgd_layer_shape.argtypes = [vp, ctypes.c_int, i32p]
        L.asgd_workspace_bytes.argtypes = [vp]
        L.asgd_workspace_bytes.restype = ctypes.c_size_t
        L.asgd_fwd_bwd.argtypes = [vp, vp, vp, vp, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, vp, vp, vp]
        L.asgd_fwd_bwd_static.argtypes = L.asgd_fwd_bwd.argtypes
        L.asgd_static_workspace_bytes.argtypes = []
        L.asgd_static_workspace_bytes.restype = ctypes.c_size_t
        L.asgd_apply_update.argtypes = [vp, vp, vp, ctypes.c_size_t, ctypes.c_float, ctypes.c_float, ctypes.c_float, vp]
        L.asgd_snapshot.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
        L.asgd_apply_update_snapshot.argtypes = [vp, vp, vp, ctypes.c_size_t, ctypes.c_float, ctypes.c_float, ctypes.c_float, vp,
                                                 ctypes.c_int, vp]
        L.asgd_train_step.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, vp, vp, ctypes.c_float,
                                      ctypes.c_float, ctypes.c_float, vp]
        L.asgd_train_step_fused.argtypes = L.asgd_train_step.argtypes
        L.asgd_debug_get.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp]
        L.asgd_profile_begin.argtypes = [vp]
        L.asgd_profile_end.argtypes = [vp, ctypes.POINTER(ProfileEntry)]
        L.asgd_schedule_generate.argtypes = [i32p, i32p, ctypes.c_int, ctypes.c_uint64, ctypes.c_int, ctypes.c_int]
        L.asgd_replay_run.argtypes = [ctypes.POINTER(vp), ctypes.c_int, vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp,
                                      i32p, i32p, ctypes.c_int, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                      ctypes.c_uint64, vp, vp, vp]
        L.asgd_replay_nsync_run.argtypes = [ctypes.POINTER(vp), ctypes.c_int, ctypes.c_int, vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                            ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp, i32p, i32p, ctypes.c_int,
                                            ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_uint64, vp, vp, vp]
        L.asgd_accumulate.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
        L.asgd_apply_update_adagrad.argtypes = [vp, vp, vp, ctypes.c_size_t, ctypes.c_float, ctypes.c_float, ctypes.c_float, vp]
        L.asgd_apply_update_adadelta.argtypes = [vp, vp, vp, vp, ctypes.c_size_t, ctypes.c_float, ctypes.c_float, ctypes.c_float, vp]
        L.asgd_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def asgd_last_error():
    return lib().asgd_last_error().decode()


def _check(rc):
    if rc < 0:
        raise AsgdError(rc, asgd_last_error())
    return rc


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def layer_descs(layers):
    """Layer tuples (see ``workloads``) -> ctypes array of asgd_layer_desc_t."""
    arr = (LayerDesc * len(layers))()
    for i, l in enumerate(layers):
        kind = l[0]
        if kind == "conv":
            arr[i] = LayerDesc(LAYER_CONV, l[1], l[2], l[3], l[4], 0.0, 0.0, 0.0, l[5] if len(l) > 5 else 1)
        elif kind == "relu":
            arr[i] = LayerDesc(LAYER_RELU, 0, 0, 0, 0, 0.0, 0.0)
        elif kind == "maxpool":
            arr[i] = LayerDesc(LAYER_MAXPOOL, 0, l[1], l[2], 0, 0.0, 0.0)
        elif kind == "fc":
            arr[i] = LayerDesc(LAYER_FC, l[1], 0, 0, 0, 0.0, 0.0)
        elif kind == "dropout":
            arr[i] = LayerDesc(LAYER_DROPOUT, 0, 0, 0, 0, float(l[1]), float(l[2]) if len(l) > 2 else 0.0)
        elif kind == "softmax_ce":
            arr[i] = LayerDesc(LAYER_SOFTMAX_CE, 0, 0, 0, 0, 0.0, 0.0)
        elif kind == "lrn":    # ("lrn", size, alpha, beta, k)
            arr[i] = LayerDesc(LAYER_LRN, 0, l[1], 0, 0, float(l[2]), float(l[3]), float(l[4]))
        else:
            raise ValueError("unknown layer kind %r" % (kind,))
    return arr


def asgd_net_create(layers, batch, in_shape, compute_dtype):
    """Returns an opaque plan handle (ctypes.c_void_p)."""
    arr = layers if isinstance(layers, ctypes.Array) else layer_descs(layers)
    h = ctypes.c_void_p(0)
    _check(lib().asgd_net_create(arr, len(arr), batch, in_shape[0], in_shape[1], in_shape[2], compute_dtype, ctypes.byref(h)))
    return h


def asgd_net_prepare(net):
    _check(lib().asgd_net_prepare(net))


def asgd_net_destroy(net):
    _check(lib().asgd_net_destroy(net))


def asgd_net_set_serial(net, on):
    _check(lib().asgd_net_set_serial(net, 1 if on else 0))


def asgd_param_count(net):
    return int(lib().asgd_param_count(net))


def asgd_param_layout(net):
    n = _check(lib().asgd_param_layout(net, None, 0))
    arr = (TensorInfo * n)()
    _check(lib().asgd_param_layout(net, arr, n))
    return [dict(layer=t.layer, kind=t.kind, w_offset=t.w_offset, w_count=t.w_count, b_offset=t.b_offset,
                 b_count=t.b_count, w_shape=tuple(t.w_shape)) for t in arr]


def asgd_layer_shape(net, layer):
    chw = (ctypes.c_int32 * 3)()
    _check(lib().asgd_layer_shape(net, layer, chw))
    return tuple(chw)


def asgd_workspace_bytes(net):
    return int(lib().asgd_workspace_bytes(net))


def asgd_fwd_bwd(net, params, images, labels, dropout_seed, step, worker, loss, grads, stream=None):
    _check(lib().asgd_fwd_bwd(net, _ptr(params), _ptr(images), _ptr(labels), dropout_seed, step, worker, _ptr(loss), _ptr(grads),
                              _stream(stream)))


def asgd_fwd_bwd_static(net, params, images, labels, dropout_seed, step, worker, loss, grads, stream=None):
    _check(lib().asgd_fwd_bwd_static(net, _ptr(params), _ptr(images), _ptr(labels), dropout_seed, step, worker, _ptr(loss), _ptr(grads),
                                     _stream(stream)))


def asgd_static_workspace_bytes():
    return int(lib().asgd_static_workspace_bytes())


def asgd_apply_update(params, momentum, grads, lr, mu, wd, stream=None, n=None):
    _check(lib().asgd_apply_update(_ptr(params), _ptr(momentum), _ptr(grads), params.numel() if n is None else n, lr, mu, wd,
                                   _stream(stream)))


def asgd_snapshot(params, worker_copy, dst_dtype, stream=None, n=None):
    _check(lib().asgd_snapshot(_ptr(params), _ptr(worker_copy), params.numel() if n is None else n, dst_dtype, _stream(stream)))


def asgd_apply_update_snapshot(params, momentum, grads, lr, mu, wd, worker_copy, dst_dtype, stream=None, n=None):
    _check(lib().asgd_apply_update_snapshot(_ptr(params), _ptr(momentum), _ptr(grads), params.numel() if n is None else n, lr, mu, wd,
                                            _ptr(worker_copy), dst_dtype, _stream(stream)))


def asgd_train_step(net, master, momentum, worker_copy, images, labels, dropout_seed, step, worker, loss, grads, lr, mu, wd, stream=None):
    _check(lib().asgd_train_step(net, _ptr(master), _ptr(momentum), _ptr(worker_copy), _ptr(images), _ptr(labels), dropout_seed, step, worker,
                                 _ptr(loss), _ptr(grads), lr, mu, wd, _stream(stream)))


def asgd_train_step_fused(net, master, momentum, worker_copy, images, labels, dropout_seed, step, worker, loss, grads, lr, mu, wd, stream=None):
    _check(lib().asgd_train_step_fused(net, _ptr(master), _ptr(momentum), _ptr(worker_copy), _ptr(images), _ptr(labels), dropout_seed, step,
                                       worker, _ptr(loss), _ptr(grads), lr, mu, wd, _stream(stream)))


def asgd_debug_get(net, what, layer, dst, stream=None):
    _check(lib().asgd_debug_get(net, what, layer, _ptr(dst), dst.numel() * dst.element_size(), _stream(stream)))


def asgd_profile_begin(net):
    _check(lib().asgd_profile_begin(net))


def asgd_profile_end(net):
    """{class name: dict(launches, ms, flops, bytes)} for the calls since asgd_profile_begin."""
    arr = (ProfileEntry * len(KERNEL_CLASSES))()
    _check(lib().asgd_profile_end(net, arr))
    return {KERNEL_CLASSES[e.kclass]: dict(launches=e.launches, ms=e.ms, flops=e.flops, bytes=e.bytes) for e in arr}


def asgd_schedule_generate(T, seed, n_workers, max_stale):
    import numpy as np
    worker = np.empty((T,), dtype=np.int32)
    rv = np.empty((T,), dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    _check(lib().asgd_schedule_generate(worker.ctypes.data_as(i32p), rv.ctypes.data_as(i32p), T, seed, n_workers, max_stale))
    return worker, rv


def asgd_replay_run(nets, params, momentum, worker_copy, worker_grads, images, labels, worker, read_version, lr, mu, wd,
                    dropout_seed, losses, log, stream=None):
    import numpy as np
    W = len(nets)
    vp = ctypes.c_void_p
    net_arr = (vp * W)(*[n.value for n in nets])
    copy_arr = (vp * W)(*[t.data_ptr() for t in worker_copy])
    grad_arr = (vp * W)(*[t.data_ptr() for t in worker_grads])
    worker = np.ascontiguousarray(worker, dtype=np.int32)
    read_version = np.ascontiguousarray(read_version, dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    _check(lib().asgd_replay_run(net_arr, W, _ptr(params), _ptr(momentum), copy_arr, grad_arr, _ptr(images), _ptr(labels),
                                 worker.ctypes.data_as(i32p), read_version.ctypes.data_as(i32p), len(worker), lr, mu, wd,
                                 dropout_seed, _ptr(losses), _ptr(log), _stream(stream)))


def asgd_replay_nsync_run(nets, n_sync, params, momentum, worker_params, worker_momentum, worker_accum, worker_copy, worker_grads, images,
                          labels, worker, read_version, lr, mu, wd, dropout_seed, losses, log, stream=None):
    import numpy as np
    W = len(nets)
    vp = ctypes.c_void_p
    arr = lambda ts: (vp * W)(*[t.data_ptr() for t in ts])
    net_arr = (vp * W)(*[n.value for n in nets])
    worker = np.ascontiguousarray(worker, dtype=np.int32)
    read_version = np.ascontiguousarray(read_version, dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    _check(lib().asgd_replay_nsync_run(net_arr, W, n_sync, _ptr(params), _ptr(momentum), arr(worker_params), arr(worker_momentum),
                                       arr(worker_accum), arr(worker_copy), arr(worker_grads), _ptr(images), _ptr(labels),
                                       worker.ctypes.data_as(i32p), read_version.ctypes.data_as(i32p), len(worker), lr, mu, wd,
                                       dropout_seed, _ptr(losses), _ptr(log), _stream(stream)))


def asgd_accumulate(accum, grads, first, stream=None, n=None):
    _check(lib().asgd_accumulate(_ptr(accum), _ptr(grads), accum.numel() if n is None else n, 1 if first else 0, _stream(stream)))


def asgd_apply_update_adagrad(params, hist, grads, lr, eps, wd, stream=None, n=None):
    _check(lib().asgd_apply_update_adagrad(_ptr(params), _ptr(hist), _ptr(grads), params.numel() if n is None else n, lr, eps, wd,
                                           _stream(stream)))


def asgd_apply_update_adadelta(params, avg_sq_grad, avg_sq_step, grads, rho, eps, wd, stream=None, n=None):
    _check(lib().asgd_apply_update_adadelta(_ptr(params), _ptr(avg_sq_grad), _ptr(avg_sq_step), _ptr(grads),
                                            params.numel() if n is None else n, rho, eps, wd, _stream(stream)))
