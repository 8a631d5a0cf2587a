"""Helpers for the GPU parity tests: run the HIP path through the C ABI and the
oracle on the same seeded inputs."""
import numpy as np
import torch

import oracle
from oracle import ops as oops
from paper_1312_6186_amd import binding as B
from paper_1312_6186_amd import workloads as wl

TOL = {B.F32: 1e-4, B.BF16: 2e-2}   # relative L2, per tensor (fp32 / bf16 compute)


def rel_l2(a, ref):
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    d = np.linalg.norm(ref)
    return np.linalg.norm(a - ref) / d if d > 0 else np.linalg.norm(a - ref)


class GpuNet:
    def __init__(self, layers, in_shape, batch, dtype):
        self.layers, self.in_shape, self.batch, self.dtype = layers, tuple(in_shape), batch, dtype
        self.net = B.asgd_net_create(layers, batch, in_shape, dtype)
        self.P = B.asgd_param_count(self.net)
        self.dev = torch.device("cuda:0")
        self.tdt = torch.bfloat16 if dtype == B.BF16 else torch.float32
        self.grads = torch.empty(self.P, dtype=torch.float32, device=self.dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.dev)
        self.copy = torch.empty(self.P, dtype=self.tdt, device=self.dev)

    def close(self):
        torch.cuda.synchronize()
        B.asgd_net_destroy(self.net)

    def to_device_images(self, images):
        img = wl.round_to_bf16(images) if self.dtype == B.BF16 else images
        return torch.from_numpy(np.ascontiguousarray(img)).to(self.dev).to(self.tdt).contiguous()

    def fwd_bwd(self, params_f32, images, labels, seed=0, step=0, worker=0):
        """params_f32: numpy or device fp32 master parameters.  Returns (loss, grads as numpy)."""
        master = params_f32 if torch.is_tensor(params_f32) else torch.from_numpy(params_f32).to(self.dev)
        B.asgd_snapshot(master, self.copy, self.dtype)
        img = self.to_device_images(images)
        lab = torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).to(self.dev)
        B.asgd_fwd_bwd(self.net, self.copy, img, lab, seed, step, worker, self.loss, self.grads)
        torch.cuda.synchronize()
        return float(self.loss.item()), self.grads.cpu().numpy()

    def debug(self, what, layer):
        """Export of layer `layer` as a numpy array of shape (B, C, H, W) (FC side: (B, F, 1, 1))."""
        shape = B.asgd_layer_shape(self.net, layer)
        dst = torch.empty((self.batch,) + shape, dtype=torch.float32 if what == B.DEBUG_OUTPUT else torch.uint8,
                          device=self.dev)
        B.asgd_debug_get(self.net, what, layer, dst)
        torch.cuda.synchronize()
        return dst.cpu().numpy()


def oracle_inputs(params_f32, images, dtype):
    """The values the HIP path actually consumes, widened to float64."""
    if dtype == B.BF16:
        return oops.bf16_to_f64(oops.snapshot_bf16(params_f32)), wl.round_to_bf16(images).astype(np.float64)
    return params_f32.astype(np.float64), images.astype(np.float64)


def compare_grads(onet, gpu_grads, ref_grads, tol, label=""):
    """Per-tensor and whole-buffer relative L2; returns the list of (name, error)."""
    errs = []
    for li, (w_off, w_shape, b_off, b_len) in sorted(onet.param_slices.items()):
        n = int(np.prod(w_shape))
        errs.append(("%s layer%d.dW" % (label, li), rel_l2(gpu_grads[w_off:w_off + n], ref_grads[w_off:w_off + n])))
        errs.append(("%s layer%d.db" % (label, li), rel_l2(gpu_grads[b_off:b_off + b_len], ref_grads[b_off:b_off + b_len])))
    errs.append(("%s all" % label, rel_l2(gpu_grads, ref_grads)))
    bad = [(n, e) for n, e in errs if not e < tol]
    assert not bad, "relative L2 above %g: %s" % (tol, bad)
    return errs


def gpu_decisions(g, layers, trace, dtype):
    """ReLU masks and pooling positions the HIP path took, checked for validity against the oracle's values.

    The two sides sum in different orders, so a pre-activation that is zero up to rounding, or two window
    elements equal up to rounding, can be decided differently; either decision is correct.  Every decision
    that differs from the oracle's is required to be such a near-tie (within the value tolerance); the caller then follows the gradient
    of the HIP path's (valid) choice.  Returns (decisions, number of differing decisions)."""
    # Values are only required to agree within TOL (relative L2), so a decision is ambiguous exactly when the
    # quantity that decides it (the pre-activation; the gap between the two largest window elements) is
    # within that tolerance of the layer's scale.
    relu_atol = pool_rtol = TOL[dtype]
    dec = {"relu": {}, "argmax": {}}
    flips = 0
    for li, l in enumerate(layers):
        if l[0] == "relu":
            pre = trace[li]["pre"]
            o_mask = pre > 0
            if layers[li + 1][0] == "dropout":
                kept = trace[li + 1]["mask"].reshape(pre.shape) == 1
                g_mask = np.where(kept, g.debug(B.DEBUG_OUTPUT, li + 1).reshape(pre.shape) > 0, o_mask)
            else:
                g_mask = g.debug(B.DEBUG_OUTPUT, li).reshape(pre.shape) > 0
            diff = g_mask != o_mask
            if diff.any():
                rms = np.sqrt(np.mean(pre ** 2))
                assert np.abs(pre[diff]).max() <= relu_atol * rms, ("ReLU decision differs away from zero", li)
                flips += int(diff.sum())
            dec["relu"][li] = g_mask
        elif l[0] == "maxpool":
            k, s = l[1], l[2]
            o_arg = trace[li]["argmax"]
            g_arg = g.debug(B.DEBUG_ARGMAX, li)
            assert g_arg.max() < k * k
            diff = g_arg != o_arg
            if diff.any():
                at_gpu = oops.maxpool_gather(trace[li - 1]["out"], g_arg, k, s)
                p = trace[li]["out"]
                rms = np.sqrt(np.mean(p ** 2))
                assert (np.abs(at_gpu - p)[diff] <= pool_rtol * np.maximum(np.abs(p)[diff], rms)).all(), \
                    ("pooling position differs although the window has a clear maximum", li)
                flips += int(diff.sum())
            dec["argmax"][li] = g_arg
    return dec, flips
