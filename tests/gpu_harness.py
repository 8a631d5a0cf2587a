"""Helpers for the GPU parity tests: run the HIP path through the C ABI and the
oracle on the same seeded inputs."""
import sys

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


def progress(capsys, msg):
    """A line on the real stdout (pytest captures the rest): the long oracle passes report when they end."""
    if capsys is None:
        print(msg)
        return
    with capsys.disabled():
        sys.stdout.write("\n    [%s]" % msg)
        sys.stdout.flush()


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


def grad_errors(onet, gpu_grads, ref_grads, label=""):
    """[(tensor name, relative L2)] per parameter tensor and over the whole flat buffer."""
    errs = []
    for li, (w_off, w_shape, b_off, b_len) in sorted(onet.param_slices.items()):
        n = int(np.prod(w_shape))
        errs.append(("%s layer%d.dW" % (label, li), rel_l2(gpu_grads[w_off:w_off + n], ref_grads[w_off:w_off + n])))
        errs.append(("%s layer%d.db" % (label, li), rel_l2(gpu_grads[b_off:b_off + b_len], ref_grads[b_off:b_off + b_len])))
    errs.append(("%s all" % label, rel_l2(gpu_grads, ref_grads)))
    return errs


def compare_grads(onet, gpu_grads, ref_grads, tol, label=""):
    """Per-tensor and whole-buffer relative L2 against `tol`; returns the list of (name, error)."""
    errs = grad_errors(onet, gpu_grads, ref_grads, label)
    bad = [(n, e) for n, e in errs if not e < tol]
    assert not bad, "relative L2 above %g: %s" % (tol, bad)
    return errs


def error_table(title, columns):
    """Text table of per-tensor errors: columns = [(heading, [(name, err)])], all over the same tensors."""
    names = [n.strip() for n, _ in columns[0][1]]
    lines = ["%s" % title, "  %-14s" % "tensor" + "".join("%22s" % h for h, _ in columns)]
    for i, n in enumerate(names):
        lines.append("  %-14s" % n + "".join("%22.3e" % col[i][1] for _, col in columns))
    return "\n".join(lines)


# How wide a near-tie may be.  The two sides sum in different orders (and, in bf16 networks, round stored
# activations that differ in the last fp32 bits to different bf16 neighbours), so the quantity that decides a ReLU
# mask or a pooling position differs between them by about the value error of that layer.  A decision of the HIP
# path that differs from the oracle's is accepted only where the oracle's own deciding quantity lies within BAND_K
# times the MEASURED relative L2 error of that layer's values (not the tolerance), never more than the tolerance
# and never less than a few fp32 roundings.
BAND_K = 8.0
BAND_FLOOR = 1e-6


def _band(err, tol):
    return min(tol, max(BAND_FLOOR, BAND_K * err))


def gpu_decisions(g, layers, trace, dtype, trace_plain=None):
    """ReLU masks and pooling positions the HIP path took, checked against the oracle.

    (1) Exactness on identical bytes: every pooling layer's positions and pooled values must equal, bit for bit,
        the oracle's pooling of the HIP path's OWN exported input (first maximum in row-major order).  ReLU masks
        of the backward pass are `stored activation > 0` by construction.
    (2) Where a decision differs from the one the oracle took on ITS values, the oracle's deciding quantity (the
        pre-activation; the gap between the window's maximum and the element the HIP path picked) must lie within
        the band derived from the measured value error of that layer (see BAND_K).
    (3) The number of differing decisions per layer is bounded.  ReLU: a handful plus half of the oracle's
        pre-activations that lie inside the band (a kernel that took every one of those the other way fails), or, if
        larger, the number of masks that differ between the oracle's own two precisions (`trace_plain`: the same
        oracle without bf16 rounding of stored activations).  Pooling: a handful plus 1e-5 of the windows in fp32; in
        bf16 a fraction of the windows that follows from the measured value error of the pool's input (see below).
    Returns (decisions, report); report["flips"] is the total, report["layers"] the per-layer detail."""
    tol = TOL[dtype]
    dec = {"relu": {}, "argmax": {}}
    report = {"flips": 0, "layers": []}
    for li, l in enumerate(layers):
        if l[0] == "relu":
            pre = trace[li]["pre"]
            o_mask = pre > 0
            lo = li + 1 if layers[li + 1][0] == "dropout" else li        # the layer whose output the group stores
            out_gpu = g.debug(B.DEBUG_OUTPUT, lo).reshape(pre.shape)
            err = rel_l2(out_gpu, trace[lo]["out"])
            if lo != li:
                kept = trace[lo]["mask"].reshape(pre.shape) == 1
                g_mask = np.where(kept, out_gpu > 0, o_mask)
            else:
                g_mask = out_gpu > 0
            rms = np.sqrt(np.mean(pre ** 2))
            band = _band(err, tol) * rms
            diff = g_mask != o_mask
            nflip = int(diff.sum())
            inside = int((np.abs(pre) <= band).sum())
            if nflip:
                assert np.abs(pre[diff]).max() <= band, ("ReLU decision differs away from zero", li, float(np.abs(pre[diff]).max()), band)
            bound = 4 + inside // 2
            if trace_plain is not None:
                bound = max(bound, int(((trace_plain[li]["pre"] > 0) != o_mask).sum()))
            assert nflip <= bound, ("too many differing ReLU decisions", li, nflip, bound)
            report["layers"].append(dict(layer=li, kind="relu", flips=nflip, bound=bound, value_err=err, band_rel=band / rms if rms > 0 else 0.0,
                                         decisions=int(pre.size)))
            report["flips"] += nflip
            dec["relu"][li] = g_mask
        elif l[0] == "maxpool":
            k, s = l[1], l[2]
            o_arg = trace[li]["argmax"]
            g_arg = g.debug(B.DEBUG_ARGMAX, li)
            assert g_arg.max() < k * k
            # (1) the kernel's positions on its own input, bit for bit
            in_gpu = g.debug(B.DEBUG_OUTPUT, li - 1).astype(np.float64)
            p_own, arg_own = oops.maxpool_fwd(in_gpu, k, s)
            np.testing.assert_array_equal(g_arg, arg_own, err_msg="pooling positions on the kernel's own input, layer %d" % li)
            np.testing.assert_array_equal(g.debug(B.DEBUG_OUTPUT, li).astype(np.float64), p_own,
                                          err_msg="pooled values on the kernel's own input, layer %d" % li)
            # (2), (3) against the oracle's positions on the oracle's values
            x_o = trace[li - 1]["out"]
            err = rel_l2(in_gpu, x_o)
            rms = np.sqrt(np.mean(x_o ** 2))
            band = 2.0 * _band(err, tol) * rms      # two elements, each off by the value error
            diff = g_arg != o_arg
            nflip = int(diff.sum())
            if nflip:
                p_o = trace[li]["out"]
                gap = p_o - oops.maxpool_gather(x_o, g_arg, k, s)      # >= 0
                allowed = np.full(p_o.shape, band)
                if dtype == B.BF16:
                    # stored activations are bf16 numbers: values that differ in their last fp32 bits can be stored one
                    # bf16 step apart, so each of the two compared elements may be off by one step of its magnitude
                    allowed += 2.0 * np.exp2(np.floor(np.log2(np.maximum(np.abs(p_o), 1e-30))) - 7)
                assert (gap[diff] <= allowed[diff]).all(), ("pooling position differs although the window has a clear maximum", li,
                                                            float(gap[diff].max()), band)
            # fp32: a handful plus 1e-5 of the windows.  bf16: about 6 % of the windows hold two maxima within one bf16
            # step of each other, and such a window flips when one of the two is stored one step apart on the two
            # sides; the fraction f of elements stored differently follows from the measured error (each contributes
            # one step, 2^-8 relative: err = sqrt(f) * 2^-8), so about 0.06 f of the windows may differ: 0.25 f allowed.
            if dtype == B.F32:
                bound = 4 + int(1e-5 * o_arg.size)
            else:
                bound = 4 + int(max(1e-5, 0.25 * (err * 256.0) ** 2) * o_arg.size)
            assert nflip <= bound, ("too many differing pooling positions", li, nflip, bound)
            report["layers"].append(dict(layer=li, kind="maxpool", flips=nflip, bound=bound, value_err=err, band_rel=band / rms if rms > 0 else 0.0,
                                         decisions=int(o_arg.size)))
            report["flips"] += nflip
            dec["argmax"][li] = g_arg
    return dec, report


def decisions_line(report):
    return "; ".join("L%d %s %d/%d (<=%d, value err %.1e, band %.1e)" % (r["layer"], r["kind"], r["flips"], r["decisions"], r["bound"],
                                                                       r["value_err"], r["band_rel"]) for r in report["layers"])
