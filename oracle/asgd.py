"""Parameter-server side of GPU A-SGD, step by step (Sections 2.2-2.3).

``replay`` is the protocol with prescribed stale reads: the server keeps the
parameter versions, update a is computed by its worker on version
``read_version[a]`` and applied to version a, giving version a+1.  Each push is
one raw minibatch-mean gradient; the server owns the momentum buffer.
"""
import numpy as np

from . import ops


def worker_copy(params, worker_dtype):
    """What a replica receives on a fetch: the fp32 parameters as they are, or
    rounded to bf16 (RNE) and widened again."""
    if worker_dtype == "f32":
        return params.astype(np.float32).astype(np.float64)
    if worker_dtype == "bf16":
        return ops.bf16_to_f64(ops.snapshot_bf16(params.astype(np.float32)))
    if worker_dtype == "f64":
        return params.copy()
    raise ValueError(worker_dtype)


def sgd_loop(net, params0, batch_fn, T, lr, mu, wd, dropout_seed=0, worker_dtype="f64", act_dtype="f64"):
    """Plain single-worker momentum SGD: T steps, step a uses batch_fn(a)."""
    w = np.array(params0, dtype=np.float64)
    v = np.zeros_like(w)
    losses = []
    for a in range(T):
        images, labels = batch_fn(a)
        loss, g, _ = net.fwd_bwd(worker_copy(w, worker_dtype), images, labels, dropout_seed, a, 0, act_dtype=act_dtype)
        ops.apply_update(w, v, g, lr, mu, wd)
        losses.append(loss)
    return w, v, losses


def replay(net, params0, worker, read_version, batch_fn, lr, mu, wd, dropout_seed=0,
           worker_dtype="f64", act_dtype="f64"):
    """A-SGD with the given schedule.  Returns final params, momentum, the loss of
    every pushed gradient and the log of (update, worker, version read)."""
    T = len(worker)
    w = np.array(params0, dtype=np.float64)
    v = np.zeros_like(w)
    versions = {0: w.copy()}
    losses, log = [], []
    for a in range(T):
        r = int(read_version[a])
        assert 0 <= r <= a
        images, labels = batch_fn(a)
        loss, g, _ = net.fwd_bwd(worker_copy(versions[r], worker_dtype), images, labels, dropout_seed, a,
                                 int(worker[a]), act_dtype=act_dtype)
        ops.apply_update(w, v, g, lr, mu, wd)
        versions[a + 1] = w.copy()
        oldest_needed = min([int(read_version[b]) for b in range(a + 1, T)] + [a + 1])
        for key in [k for k in versions if k < oldest_needed]:
            del versions[key]
        losses.append(loss)
        log.append((a, int(worker[a]), r))
    return w, v, losses, np.array(log, dtype=np.int32)
