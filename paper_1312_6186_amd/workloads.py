"""Seeded synthetic workloads: network descriptors and input generators.

This module holds none of the method's arithmetic.  It only names the network
configurations and draws the random inputs (images, labels, initial
parameters) that both the HIP path and the test oracle are fed, so that the two
see identical bytes.  Synthetic N(0,1) images of the crop shape and uniform
labels stand in for the ILSVRC-2012 data the paper trains on (Section 1).

A network is a list of layer tuples:
    ("conv", cout, k, stride, pad[, groups])  ("relu",)  ("maxpool", k, stride)
    ("fc", out)  ("dropout", p)  ("softmax_ce",)  ("lrn", size, alpha, beta, k)
"""
import numpy as np


LRN = ("lrn", 5, 1e-4, 0.75, 2.0)   # the constants of the cited architecture (Krizhevsky et al. 2012, Section 3.3)


def _conv_block(cout, k, stride, pad, pool=None, lrn=False, groups=1):
    block = [("conv", cout, k, stride, pad) + ((groups,) if groups > 1 else ()), ("relu",)]
    if lrn:
        block.append(LRN)
    if pool:
        block.append(("maxpool",) + pool)
    return block


TINY = {
    "name": "tiny", "in_shape": (1, 28, 28), "batch": 8, "classes": 10,
    "layers": _conv_block(8, 5, 1, 2, (2, 2)) + [("fc", 10), ("softmax_ce",)],
    "lr": 0.01, "mu": 0.9, "wd": 0.0, "seeds": {"data": 1001, "init": 2001, "dropout": 0},
}

SMALL = {
    "name": "small", "in_shape": (3, 32, 32), "batch": 128, "classes": 10,
    "layers": (_conv_block(32, 5, 1, 2, (3, 2)) + _conv_block(32, 5, 1, 2, (3, 2))
               + _conv_block(64, 5, 1, 2, (3, 2))
               + [("fc", 64), ("relu",), ("dropout", 0.5), ("fc", 10), ("softmax_ce",)]),
    "lr": 0.01, "mu": 0.9, "wd": 0.0, "seeds": {"data": 1002, "init": 2002, "dropout": 3002},
}

ALEXNET = {
    "name": "alexnet", "in_shape": (3, 224, 224), "batch": 128, "classes": 1000,
    "layers": (_conv_block(96, 11, 4, 2, (3, 2)) + _conv_block(256, 5, 1, 2, (3, 2))
               + _conv_block(384, 3, 1, 1) + _conv_block(384, 3, 1, 1) + _conv_block(256, 3, 1, 1, (3, 2))
               + [("fc", 4096), ("relu",), ("dropout", 0.5), ("fc", 4096), ("relu",), ("dropout", 0.5),
                  ("fc", 1000), ("softmax_ce",)]),
    "lr": 0.01, "mu": 0.9, "wd": 5e-4, "seeds": {"data": 1003, "init": 2003, "dropout": 3003},
}

# the same net with the response normalisation of the cited architecture after conv1 and conv2 (before the pools)
ALEXNET_LRN = dict(ALEXNET, name="alexnet_lrn",
                   layers=(_conv_block(96, 11, 4, 2, (3, 2), lrn=True) + _conv_block(256, 5, 1, 2, (3, 2), lrn=True)
                           + ALEXNET["layers"][6:]))

# the cited architecture in full: response normalisation after conv1 / conv2 and two-column (grouped) conv2, conv4, conv5
ALEXNET_FULL = dict(ALEXNET, name="alexnet_full",
                    layers=(_conv_block(96, 11, 4, 2, (3, 2), lrn=True) + _conv_block(256, 5, 1, 2, (3, 2), lrn=True, groups=2)
                            + _conv_block(384, 3, 1, 1) + _conv_block(384, 3, 1, 1, groups=2)
                            + _conv_block(256, 3, 1, 1, (3, 2), groups=2) + ALEXNET["layers"][13:]))

CONFIGS = {"tiny": TINY, "small": SMALL, "alexnet": ALEXNET, "alexnet_lrn": ALEXNET_LRN, "alexnet_full": ALEXNET_FULL}


def param_shapes(layers, in_shape):
    """[(layer index, weight shape, bias length, fan_in)] in flat-buffer order."""
    shape = tuple(in_shape)
    out = []
    for li, l in enumerate(layers):
        if l[0] == "conv":
            cout, k, s, p = l[1:5]
            groups = l[5] if len(l) > 5 else 1
            c, h, w = shape
            out.append((li, (cout, c // groups, k, k), cout, (c // groups) * k * k))
            shape = (cout, (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1)
        elif l[0] == "maxpool":
            _, k, s = l
            c, h, w = shape
            shape = (c, (h - k) // s + 1, (w - k) // s + 1)
        elif l[0] == "fc":
            nin = int(np.prod(shape))
            out.append((li, (l[1], nin), l[1], nin))
            shape = (l[1],)
    return out


def param_count(layers, in_shape):
    return sum(int(np.prod(ws)) + bl for _, ws, bl, _ in param_shapes(layers, in_shape))


def make_params(layers, in_shape, seed):
    """He-normal weights N(0, 2/fan_in), zero biases, as one flat fp32 vector."""
    rng = np.random.default_rng(seed)
    parts = []
    for _, wshape, blen, fan_in in param_shapes(layers, in_shape):
        n = int(np.prod(wshape))
        parts.append((rng.standard_normal(n, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))))
        parts.append(np.zeros(blen, dtype=np.float32))
    return np.concatenate(parts)


def make_batch(in_shape, batch, classes, seed):
    """N(0,1) fp32 images [B,C,H,W] and uniform int32 labels [B]."""
    rng = np.random.default_rng(seed)
    images = rng.standard_normal((batch,) + tuple(in_shape), dtype=np.float32)
    labels = rng.integers(0, classes, size=(batch,), dtype=np.int32)
    return images, labels


def round_to_bf16(a):
    """Round an fp32 array to the nearest bf16-representable fp32 values (ties to even)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000))
    return r.view(np.float32).reshape(a.shape)
