"""Parameter-server side of GPU A-SGD, step by step (Sections 2.2-2.3).

``replay`` is the protocol with prescribed stale reads: the server keeps the
parameter versions, update a is computed by its worker on version
``read_version[a]`` and applied to version a, giving version a+1.  Each push is
one raw minibatch-mean gradient; the server owns the momentum buffer.

``replay_nsync`` is the regime the paper runs (Section 2.3, n_fetch = n_push =
n_sync): a replica updates its own parameters on its GPU for n_sync steps
between two exchanges with the server.
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
           worker_dtype="f64", act_dtype="f64", decisions_fn=None):
    """A-SGD with the given schedule.  Returns final params, momentum, the loss of
    every pushed gradient and the log of (update, worker, version read).
    ``decisions_fn(a, worker_params, images, labels)``, if given, may return the
    ReLU masks / pooling positions to use for update a (the ``decisions`` argument
    of ``OracleNet.fwd_bwd``; None = the oracle's own): a caller that has checked
    that another valid choice among near-ties was taken asks for its gradient.
    The protocol and the arithmetic are the same either way."""
    T = len(worker)
    w = np.array(params0, dtype=np.float64)
    v = np.zeros_like(w)
    versions = {0: w.copy()}
    losses, log = [], []
    for a in range(T):
        r = int(read_version[a])
        assert 0 <= r <= a
        images, labels = batch_fn(a)
        wc = worker_copy(versions[r], worker_dtype)
        dec = decisions_fn(a, wc, images, labels) if decisions_fn is not None else None
        loss, g, _ = net.fwd_bwd(wc, images, labels, dropout_seed, a, int(worker[a]), act_dtype=act_dtype, decisions=dec)
        ops.apply_update(w, v, g, lr, mu, wd)
        versions[a + 1] = w.copy()
        oldest_needed = min([int(read_version[b]) for b in range(a + 1, T)] + [a + 1])
        for key in [k for k in versions if k < oldest_needed]:
            del versions[key]
        losses.append(loss)
        log.append((a, int(worker[a]), r))
    return w, v, losses, np.array(log, dtype=np.int32)


def replay_nsync(net, params0, worker, read_version, batch_fn, n_sync, lr, mu, wd, dropout_seed=0,
                 worker_dtype="f64", act_dtype="f64"):
    """A-SGD with n_fetch = n_push = n_sync (Section 2.3).

    Reading of the paper's one sentence on it: cycle a belongs to replica
    worker[a].  The replica fetches version read_version[a] of the server's
    parameters into its own fp32 parameters, then runs n_sync ordinary
    momentum-SGD steps on them (same rule and hyper-parameters as the server; its
    own momentum buffer, zero at the start and kept across fetches), computing
    each gradient on its parameters as it holds them for compute (worker_dtype).
    It pushes the SUM of those n_sync minibatch gradients, which the server
    applies as one gradient, giving version a+1.  Minibatch i of cycle a is
    batch_fn(a, i); its dropout step is a*n_sync + i.  n_sync = 1 is ``replay``.

    Returns final server params and momentum, the losses [T][n_sync], the log of
    (update, worker, version read) and the replicas' (params, momentum)."""
    T = len(worker)
    W = int(max(worker)) + 1 if T else 0
    w = np.array(params0, dtype=np.float64)
    v = np.zeros_like(w)
    versions = {0: w.copy()}
    local_w = [None] * W
    local_v = [np.zeros_like(w) for _ in range(W)]
    losses, log = [], []
    for a in range(T):
        r, k = int(read_version[a]), int(worker[a])
        assert 0 <= r <= a
        # fetch: fp32 values of the server's parameters
        local_w[k] = versions[r].astype(np.float32).astype(np.float64) if worker_dtype != "f64" else versions[r].copy()
        pushed = np.zeros_like(w)
        row = []
        for i in range(n_sync):
            images, labels = batch_fn(a, i)
            loss, g, _ = net.fwd_bwd(worker_copy(local_w[k], worker_dtype), images, labels, dropout_seed,
                                     a * n_sync + i, k, act_dtype=act_dtype)
            pushed += g
            ops.apply_update(local_w[k], local_v[k], g, lr, mu, wd)
            row.append(loss)
        ops.apply_update(w, v, pushed, lr, mu, wd)
        versions[a + 1] = w.copy()
        oldest_needed = min([int(read_version[b]) for b in range(a + 1, T)] + [a + 1])
        for key in [q for q in versions if q < oldest_needed]:
            del versions[key]
        losses.append(row)
        log.append((a, k, r))
    return w, v, losses, np.array(log, dtype=np.int32), list(zip(local_w, local_v))
