"""The convnet's minibatch gradient, composed from the oracle's layer functions.

A network is a list of layer tuples:
    ("conv", cout, k, stride, pad)  ("relu",)  ("maxpool", k, stride)
    ("fc", out)  ("dropout", p[, scale])  ("softmax_ce",)
The flat parameter vector holds, for each conv/fc layer in order, the weights
(conv [cout,cin,k,k]; fc [out,in] with in = c*H*W + h*W + w) followed by the bias.
Section 2 of the paper defines the unit of work: the gradient of the objective
over one minibatch.
"""
import numpy as np

from . import ops


class OracleNet:
    def __init__(self, layers, in_shape):
        self.layers = [tuple(l) for l in layers]
        self.in_shape = tuple(in_shape)
        assert self.layers and self.layers[-1][0] == "softmax_ce"
        shape = self.in_shape  # (C,H,W) or (F,)
        self.shapes = []       # output shape of each layer
        self.param_slices = {}  # layer index -> (w_off, w_shape, b_off, b_len)
        off = 0
        for li, l in enumerate(self.layers):
            kind = l[0]
            if kind == "conv":
                cout, k, s, p = l[1:5]
                groups = l[5] if len(l) > 5 else 1       # ("conv", cout, k, stride, pad[, groups])
                c, h, w = shape
                ho, wo = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
                assert ho > 0 and wo > 0 and c % groups == 0 and cout % groups == 0
                wshape = (cout, c // groups, k, k)
                self.param_slices[li] = (off, wshape, off + int(np.prod(wshape)), cout)
                off += int(np.prod(wshape)) + cout
                shape = (cout, ho, wo)
            elif kind == "maxpool":
                _, k, s = l
                c, h, w = shape
                ho, wo = (h - k) // s + 1, (w - k) // s + 1
                assert ho > 0 and wo > 0
                shape = (c, ho, wo)
            elif kind == "fc":
                nin = int(np.prod(shape))
                wshape = (l[1], nin)
                self.param_slices[li] = (off, wshape, off + l[1] * nin, l[1])
                off += l[1] * nin + l[1]
                shape = (l[1],)
            elif kind in ("relu", "dropout", "softmax_ce", "lrn"):
                pass
            else:
                raise ValueError(kind)
            self.shapes.append(shape)
        self.param_count = off
        self.num_classes = int(np.prod(shape))

    def split(self, flat, li):
        w_off, w_shape, b_off, b_len = self.param_slices[li]
        n = int(np.prod(w_shape))
        return flat[w_off:w_off + n].reshape(w_shape), flat[b_off:b_off + b_len]

    def fwd_bwd(self, params, images, labels, dropout_seed=0, step=0, worker=0, want_grads=True,
                masks=None, act_dtype="f64", decisions=None):
        """Returns (loss, grads, trace).  ``trace[li]`` holds what layer li produced
        ("out", and "argmax" / "mask" where they exist); ``trace["dx"][li]`` the
        gradient w.r.t. that layer's input.  ``masks`` overrides the generated
        dropout masks (dict layer index -> uint8 array), for tests.
        ``act_dtype="bf16"`` models a network that stores its activations in bf16:
        every stored activation (the output of a conv or fc layer after its ReLU /
        dropout, except the final logits) is rounded to bf16, so that pooling
        positions and ReLU masks are decided on the stored values.
        ``decisions`` = {"relu": {li: bool array}, "argmax": {li: uint8 array}} fixes
        the ReLU masks / pooling positions of those layers instead of deriving them:
        a unit whose input is zero up to rounding, or a window with two maxima equal
        up to rounding, can validly go either way, and the caller (having checked
        that validity) asks for the gradient of one particular choice."""
        dec_relu = (decisions or {}).get("relu", {})
        dec_arg = (decisions or {}).get("argmax", {})
        params = np.ascontiguousarray(params, dtype=np.float64)
        assert params.shape == (self.param_count,)
        x = np.ascontiguousarray(images, dtype=np.float64)
        N = x.shape[0]
        assert x.shape[1:] == self.in_shape
        trace = {}
        inputs = []
        for li, l in enumerate(self.layers):
            kind = l[0]
            inputs.append(x)
            t = {}
            if kind == "conv":
                w, b = self.split(params, li)
                groups = l[5] if len(l) > 5 else 1
                if groups == 1:
                    x = ops.conv_fwd(x, w, b, l[3], l[4])
                else:
                    # grouped ("two-column") convolution: group g maps input channels [g*Cg, (g+1)*Cg) to output
                    # channels [g*Og, (g+1)*Og) and is an ordinary convolution of those slices
                    cg, og = x.shape[1] // groups, w.shape[0] // groups
                    x = np.concatenate([ops.conv_fwd(x[:, g * cg:(g + 1) * cg], w[g * og:(g + 1) * og], b[g * og:(g + 1) * og],
                                                     l[3], l[4]) for g in range(groups)], axis=1)
            elif kind == "relu":
                t["pre"] = x
                if li in dec_relu:
                    t["relu_mask"] = np.asarray(dec_relu[li], dtype=bool).reshape(x.shape)
                    x = np.where(t["relu_mask"], x, 0.0)
                else:
                    x = ops.relu_fwd(x)
            elif kind == "maxpool":
                if li in dec_arg:
                    t["argmax"] = np.ascontiguousarray(dec_arg[li], dtype=np.uint8)
                    x = ops.maxpool_gather(x, t["argmax"], l[1], l[2])
                else:
                    x, t["argmax"] = ops.maxpool_fwd(x, l[1], l[2])
            elif kind == "lrn":   # ("lrn", size, alpha, beta, k)
                x = ops.lrn_fwd(x, l[1], l[2], l[3], l[4])
            elif kind == "fc":
                w, b = self.split(params, li)
                x = ops.fc_fwd(x.reshape(N, -1), w, b)
            elif kind == "dropout":
                p = l[1]
                scale = l[2] if len(l) > 2 else 1.0
                if masks is not None and li in masks:
                    m = np.ascontiguousarray(masks[li], dtype=np.uint8).reshape(-1)
                else:
                    m = ops.dropout_mask(x.size, dropout_seed, step, worker, li, p)
                t["mask"] = m.reshape(x.shape)
                x = ops.dropout_apply(x, m, scale)
            elif kind == "softmax_ce":
                loss, dz = ops.softmax_ce(x.reshape(N, -1), labels, want_grad=want_grads)
                t["dz"] = dz
            if act_dtype == "bf16" and kind != "softmax_ce":
                nxt = self.layers[li + 1][0]
                stored = ((kind in ("conv", "fc") and nxt not in ("relu", "softmax_ce"))
                          or (kind == "relu" and nxt != "dropout") or kind in ("dropout", "lrn"))
                if stored:
                    x = ops.round_bf16(x)
            t["out"] = x
            trace[li] = t
        if not want_grads:
            return loss, None, trace

        grads = np.zeros((self.param_count,))
        d = dz
        trace["dx"] = {}
        for li in range(len(self.layers) - 1, -1, -1):
            l = self.layers[li]
            kind = l[0]
            xin = inputs[li]
            if kind == "softmax_ce":
                pass
            elif kind == "dropout":
                scale = l[2] if len(l) > 2 else 1.0
                d = ops.dropout_apply(d, trace[li]["mask"].reshape(-1), scale).reshape(xin.shape)
            elif kind == "relu":
                # the mask is taken on the stored ReLU output, which is positive exactly where the input was
                # (a positive input may only round to zero in bf16 when it is below the smallest bf16 subnormal)
                if li in dec_relu:
                    d = np.where(trace[li]["relu_mask"], d.reshape(xin.shape), 0.0)
                else:
                    d = ops.relu_bwd(trace[li]["out"] if act_dtype == "bf16" else xin, d.reshape(xin.shape))
            elif kind == "maxpool":
                d = ops.maxpool_bwd(d.reshape(trace[li]["out"].shape), trace[li]["argmax"], xin.shape[2:],
                                    l[1], l[2])
            elif kind == "lrn":
                d = ops.lrn_bwd(xin, d.reshape(xin.shape), l[1], l[2], l[3], l[4])
            elif kind == "fc":
                w, b = self.split(params, li)
                w_off, w_shape, b_off, b_len = self.param_slices[li]
                dx, dw, db = ops.fc_bwd(xin.reshape(N, -1), w, d.reshape(N, -1), need_dx=li > 0)
                grads[w_off:w_off + dw.size] = dw.reshape(-1)
                grads[b_off:b_off + b_len] = db
                d = dx.reshape(xin.shape) if dx is not None else None
            elif kind == "conv":
                w, b = self.split(params, li)
                w_off, w_shape, b_off, b_len = self.param_slices[li]
                dy = d.reshape(trace[li]["out"].shape)
                groups = l[5] if len(l) > 5 else 1
                if groups == 1:
                    dw, db = ops.conv_bwd_weight(xin, dy, l[2], l[3], l[4])
                    d = ops.conv_bwd_data(dy, w, xin.shape[2:], l[3], l[4]) if li > 0 else None
                else:
                    cg, og = xin.shape[1] // groups, w.shape[0] // groups
                    parts = [ops.conv_bwd_weight(xin[:, g * cg:(g + 1) * cg], dy[:, g * og:(g + 1) * og], l[2], l[3], l[4])
                             for g in range(groups)]
                    dw = np.concatenate([pw for pw, _ in parts], axis=0)
                    db = np.concatenate([pb for _, pb in parts])
                    d = np.concatenate([ops.conv_bwd_data(dy[:, g * og:(g + 1) * og], w[g * og:(g + 1) * og], xin.shape[2:], l[3], l[4])
                                        for g in range(groups)], axis=1) if li > 0 else None
                grads[w_off:w_off + dw.size] = dw.reshape(-1)
                grads[b_off:b_off + b_len] = db
            trace["dx"][li] = d
        return loss, grads, trace
