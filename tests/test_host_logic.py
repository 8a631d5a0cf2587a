"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
declared symbol, plans networks, reports shapes / parameter layout and rejects
bad arguments with error codes."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1312_6186_amd import binding as B
from paper_1312_6186_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "asgd.h")).read()
    declared = set(re.findall(r"\b(asgd_[a-z_]+)\s*\(", header))
    declared -= {"asgd_net"}
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None


@pytest.mark.parametrize("cfg", [wl.TINY, wl.SMALL, wl.ALEXNET])
def test_plan_matches_the_workload_description(cfg):
    for dt in (B.F32, B.BF16):
        net = B.asgd_net_create(cfg["layers"], cfg["batch"], cfg["in_shape"], dt)
        try:
            assert B.asgd_param_count(net) == wl.param_count(cfg["layers"], cfg["in_shape"])
            layout = B.asgd_param_layout(net)
            ref = wl.param_shapes(cfg["layers"], cfg["in_shape"])
            assert len(layout) == len(ref)
            off = 0
            for t, (li, wshape, blen, _) in zip(layout, ref):
                assert t["layer"] == li and t["w_offset"] == off and t["w_count"] == int(np.prod(wshape))
                assert t["w_shape"][:len(wshape)] == tuple(wshape)
                off += t["w_count"]
                assert t["b_offset"] == off and t["b_count"] == blen
                off += blen
            assert B.asgd_workspace_bytes(net) > 0
        finally:
            B.asgd_net_destroy(net)


def test_full_cited_architecture_has_the_published_parameter_count():
    cfg = wl.ALEXNET_FULL
    net = B.asgd_net_create(cfg["layers"], 2, cfg["in_shape"], B.BF16)
    try:
        assert B.asgd_param_count(net) == 60965224 == wl.param_count(cfg["layers"], cfg["in_shape"])
        lay = {t["layer"]: t for t in B.asgd_param_layout(net)}
        assert lay[4]["w_shape"] == (256, 48, 5, 5) and lay[10]["w_shape"] == (384, 192, 3, 3) and lay[12]["w_shape"] == (256, 192, 3, 3)
    finally:
        B.asgd_net_destroy(net)


def test_alexnet_shapes():
    net = B.asgd_net_create(wl.ALEXNET["layers"], 128, (3, 224, 224), B.BF16)
    shapes = [B.asgd_layer_shape(net, i) for i in range(len(wl.ALEXNET["layers"]))]
    assert shapes[0] == (96, 55, 55) and shapes[2] == (96, 27, 27) and shapes[5] == (256, 13, 13)
    assert shapes[12] == (256, 6, 6) and shapes[13] == (4096, 1, 1) and shapes[-1] == (1000, 1, 1)
    B.asgd_net_destroy(net)


def _rc(layers, batch=4, in_shape=(3, 16, 16), dt=B.F32):
    arr = B.layer_descs(layers)
    h = ctypes.c_void_p(0)
    rc = B.lib().asgd_net_create(arr, len(arr), batch, in_shape[0], in_shape[1], in_shape[2], dt, ctypes.byref(h))
    if rc == 0:
        B.asgd_net_destroy(h)
    return rc


def test_bad_descriptors_are_rejected_with_codes():
    ok = [("conv", 8, 3, 1, 1), ("relu",), ("maxpool", 2, 2), ("fc", 10), ("softmax_ce",)]
    assert _rc(ok) == B.OK
    assert _rc(ok[:-1]) == B.ESHAPE                                   # no loss layer
    assert _rc([("relu",)] + ok) == B.ESHAPE                          # ReLU with nothing to fuse into
    assert _rc([("conv", 8, 32, 1, 0), ("fc", 10), ("softmax_ce",)]) == B.ESHAPE  # filter larger than image
    assert _rc([("conv", 8, 3, 1, 1), ("maxpool", 20, 2), ("fc", 10), ("softmax_ce",)]) == B.ESHAPE
    assert _rc([("conv", 3, 3, 1, 0), ("fc", 10), ("softmax_ce",)], in_shape=(3, 5, 5)) == B.ESHAPE  # fan-in 27
    assert _rc([("fc", 16), ("dropout", 0.5), ("fc", 10), ("softmax_ce",)]) == B.ESHAPE       # dropout needs FC+ReLU
    assert _rc([("fc", 16), ("relu",), ("dropout", 1.0), ("fc", 10), ("softmax_ce",)]) == B.ESHAPE
    lrn = [("conv", 8, 3, 1, 1), ("relu",), ("lrn", 5, 1e-4, 0.75, 2.0), ("maxpool", 2, 2), ("fc", 10), ("softmax_ce",)]
    assert _rc(lrn) == B.OK
    assert _rc([lrn[0]] + lrn[2:]) == B.ESHAPE                        # LRN needs CONV + RELU right before it
    assert _rc(lrn[:2] + [lrn[3], lrn[2]] + lrn[4:]) == B.ESHAPE      # not after a pool
    assert _rc(lrn[:2] + [("lrn", 4, 1e-4, 0.75, 2.0)] + lrn[3:]) == B.ESHAPE    # even window
    assert _rc(lrn[:2] + [("lrn", 11, 1e-4, 0.75, 2.0)] + lrn[3:]) == B.ESHAPE   # window above 9
    assert _rc(lrn[:2] + [("lrn", 5, 1e-4, 0.75, 0.0)] + lrn[3:]) == B.ESHAPE    # bias must be positive
    grp = [("conv", 16, 3, 1, 1), ("relu",), ("conv", 32, 3, 1, 1, 2), ("relu",), ("maxpool", 2, 2), ("fc", 10), ("softmax_ce",)]
    assert _rc(grp) == B.OK
    assert _rc(grp[:2] + [("conv", 32, 3, 1, 1, 4)] + grp[3:]) == B.ESHAPE      # 4 input channels per group: not a multiple of 8
    assert _rc(grp[:2] + [("conv", 24, 3, 1, 1, 2)] + grp[3:]) == B.ESHAPE      # 12 output channels per group
    assert _rc(grp[:2] + [("conv", 32, 3, 1, 1, 3)] + grp[3:]) == B.ESHAPE      # 16 does not divide by 3
    assert _rc(ok, batch=0) == B.ESHAPE
    assert _rc(ok, dt=7) == B.EINVAL
    assert "dtype" in B.asgd_last_error()
    h = ctypes.c_void_p(0)
    assert B.lib().asgd_net_create(None, 3, 1, 1, 1, 1, 0, ctypes.byref(h)) == B.EINVAL
    bad = (B.LayerDesc * 1)(B.LayerDesc(99, 0, 0, 0, 0, 0.0, 0.0))
    assert B.lib().asgd_net_create(bad, 1, 1, 1, 8, 8, 0, ctypes.byref(h)) == B.EINVAL


def test_null_and_misaligned_pointers_are_rejected_before_any_gpu_work():
    L = B.lib()
    net = B.asgd_net_create(wl.TINY["layers"], 8, (1, 28, 28), B.F32)
    vp = ctypes.c_void_p
    assert L.asgd_fwd_bwd(net, vp(0), vp(16), vp(16), 0, 0, 0, vp(16), vp(16), vp(0)) == B.EINVAL
    assert L.asgd_fwd_bwd(net, vp(4), vp(16), vp(16), 0, 0, 0, vp(16), vp(16), vp(0)) == B.EALIGN
    assert L.asgd_apply_update(vp(0), vp(16), vp(16), 10, 0.1, 0.9, 0.0, vp(0)) == B.EINVAL
    assert L.asgd_apply_update(vp(0), vp(0), vp(0), 0, 0.1, 0.9, 0.0, vp(0)) == B.OK          # nothing to do
    assert L.asgd_apply_update(vp(2), vp(16), vp(16), 10, 0.1, 0.9, 0.0, vp(0)) == B.EALIGN
    assert L.asgd_snapshot(vp(16), vp(16), 10, 5, vp(0)) == B.EINVAL
    assert L.asgd_snapshot(vp(0), vp(16), 10, B.BF16, vp(0)) == B.EINVAL
    assert L.asgd_debug_get(net, 0, 1, vp(16), 1 << 20, vp(0)) == B.EINVAL                     # nothing has run yet
    assert L.asgd_layer_shape(net, 99, (ctypes.c_int32 * 3)()) == B.EINVAL
    assert B.asgd_param_count(vp(0)) == 0
    B.asgd_net_destroy(net)
    assert L.asgd_net_destroy(vp(0)) == B.OK


def test_schedule_generator_agrees_with_definition_and_rejects_bad_arguments():
    MASK = (1 << 64) - 1

    def mix(z):
        z ^= z >> 30; z = (z * 0xBF58476D1CE4E5B9) & MASK
        z ^= z >> 27; z = (z * 0x94D049BB133111EB) & MASK
        return z ^ (z >> 31)

    worker, rv = B.asgd_schedule_generate(64, 4005, 4, 3)
    for a in range(64):
        assert worker[a] == a % 4 and rv[a] == a - min(a, (mix((mix(4005) + a) & MASK) >> 32) % 4)
    i32p = ctypes.POINTER(ctypes.c_int32)
    w = np.zeros(4, np.int32)
    assert B.lib().asgd_schedule_generate(w.ctypes.data_as(i32p), w.ctypes.data_as(i32p), 4, 1, 4, 4) == B.EINVAL
    assert B.lib().asgd_schedule_generate(None, None, 4, 1, 4, 3) == B.EINVAL


def test_replay_rejects_impossible_schedules_without_a_gpu():
    L = B.lib()
    vp = ctypes.c_void_p
    nets = [B.asgd_net_create(wl.TINY["layers"], 8, (1, 28, 28), B.F32) for _ in range(2)]
    net_arr = (vp * 2)(*[n.value for n in nets])
    bufs = (vp * 2)(16, 32)
    i32p = ctypes.POINTER(ctypes.c_int32)

    def run(worker, rv):
        w = np.array(worker, np.int32); r = np.array(rv, np.int32)
        return L.asgd_replay_run(net_arr, 2, vp(16), vp(16), bufs, bufs, vp(16), vp(16), w.ctypes.data_as(i32p),
                                 r.ctypes.data_as(i32p), len(worker), 0.1, 0.9, 0.0, 0, vp(16), vp(16), vp(0))

    assert run([0, 1, 0], [0, 0, 3]) == B.EINVAL      # reads a version that does not exist yet
    assert run([0, 1, 0], [0, 0, 0]) == B.EINVAL      # worker 0 reads before its own push 0 was applied
    assert run([0, 5], [0, 0]) == B.EINVAL            # no such worker
    for n in nets:
        B.asgd_net_destroy(n)
