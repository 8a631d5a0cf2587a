"""The entry point that allocates nothing (asgd_fwd_bwd_static) against asgd_fwd_bwd, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_1312_6186_amd import binding as B
from paper_1312_6186_amd import workloads as wl

DEV = "cuda:0"


def test_oversized_plan_is_refused_without_touching_the_gpu():
    cfg = wl.ALEXNET
    net = B.asgd_net_create(cfg["layers"], 128, cfg["in_shape"], B.BF16)
    try:
        assert B.asgd_workspace_bytes(net) > B.asgd_static_workspace_bytes() == 64 << 20
        import ctypes
        dummy = ctypes.c_void_p(4096)     # never dereferenced: the size check comes before any device work
        rc = B.lib().asgd_fwd_bwd_static(net, dummy, dummy, dummy, 0, 0, 0, dummy, dummy, ctypes.c_void_p(0))
        assert rc == B.ENOMEM and "static workspace" in B.asgd_last_error()
    finally:
        B.asgd_net_destroy(net)


def _case(cfg, batch, dtype, seed):
    layers, in_shape = cfg["layers"], cfg["in_shape"]
    tdt = torch.bfloat16 if dtype == B.BF16 else torch.float32
    params = torch.from_numpy(wl.make_params(layers, in_shape, seed)).to(DEV)
    images_np, labels_np = wl.make_batch(in_shape, batch, cfg["classes"], seed + 1)
    images = torch.from_numpy(images_np).to(DEV).to(tdt).contiguous()
    labels = torch.from_numpy(labels_np).to(DEV)
    copy = torch.empty(params.numel(), dtype=tdt, device=DEV)
    B.asgd_snapshot(params, copy, dtype)
    return layers, in_shape, copy, images, labels


@pytest.mark.gpu
def test_static_entry_point_matches_fwd_bwd_on_two_calls_in_a_row():
    """Two calls in a row on the shared static workspace, the second on a smaller plan (whose tensors then lie over
    what the first call left), each compared bit for bit with asgd_fwd_bwd on a plan with its own workspace."""
    cases = [(wl.SMALL, 32, B.F32, 11), (wl.TINY, 8, B.F32, 12), (wl.SMALL, 16, B.BF16, 13)]
    stat_nets, outs = [], []
    try:
        for cfg, batch, dtype, seed in cases:            # the static calls back to back, nothing between them
            layers, in_shape, copy, images, labels = _case(cfg, batch, dtype, seed)
            net = B.asgd_net_create(layers, batch, in_shape, dtype)
            stat_nets.append(net)
            assert B.asgd_workspace_bytes(net) <= B.asgd_static_workspace_bytes()
            loss = torch.full((1,), float("nan"), device=DEV)
            grads = torch.full((B.asgd_param_count(net),), float("nan"), device=DEV)
            B.asgd_fwd_bwd_static(net, copy, images, labels, 77, 5, 2, loss, grads)
            outs.append((loss, grads, (copy, images, labels)))
        torch.cuda.synchronize()
        for (cfg, batch, dtype, seed), (loss, grads, (copy, images, labels)) in zip(cases, outs):
            net = B.asgd_net_create(cfg["layers"], batch, cfg["in_shape"], dtype)
            try:
                ref_loss = torch.zeros(1, device=DEV)
                ref_grads = torch.empty_like(grads)
                B.asgd_fwd_bwd(net, copy, images, labels, 77, 5, 2, ref_loss, ref_grads)
                torch.cuda.synchronize()
                assert np.isfinite(ref_grads.cpu().numpy()).all()
                assert loss.cpu().numpy().tobytes() == ref_loss.cpu().numpy().tobytes()
                assert grads.cpu().numpy().tobytes() == ref_grads.cpu().numpy().tobytes()
            finally:
                torch.cuda.synchronize()
                B.asgd_net_destroy(net)
    finally:
        torch.cuda.synchronize()
        for net in stat_nets:
            B.asgd_net_destroy(net)
