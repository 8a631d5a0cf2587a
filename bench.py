"""Benchmark of the GPU A-SGD hot path on one MI355X.

A step is one worker's whole cycle on one minibatch of synthetic data resident
in HBM: fwd+bwd (the minibatch gradient on the worker's copy of the parameters),
the server's momentum / weight-decay update, and the fetch of the updated fp32
parameters into the worker's copy (the last two in one pass,
asgd_apply_update_snapshot).  Prints ONE JSON line: images/sec, the roofline
fraction of the dominant kernel class (timed with HIP events on the stream the
kernels run on, in a second pass that runs the kernels one after the other;
the timed pass overlaps the parameter-gradient kernels with the data path),
the per-class table, and the CPU oracle timed on a bounded sample.

    python bench.py [--steps K] [--warmup W] [--workload alexnet_bf16_bs128]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: (batch, compute dtype)
    "alexnet_bf16_bs128": (128, "bf16"),   # the headline: AlexNet-style single column, bf16 MFMA, fp32 master weights
    "alexnet_f32_bs128": (128, "f32"),
    "alexnet_bf16_bs256": (256, "bf16"),
    "alexnet_lrn_bf16_bs128": (128, "bf16"),  # with the response normalisation of the cited architecture after conv1, conv2
    "alexnet_full_bf16_bs128": (128, "bf16"),  # the cited architecture in full: LRN and two-column conv2 / conv4 / conv5
    # A-SGD on one GPU: 4 workers as concurrent streams, batch 32 each, snapshots up to 3 updates stale;
    # a step is one pushed gradient (snapshot + fwd_bwd + server update)
    "asgd_4x32_bf16": (32, "bf16"),
    # the same replicas in the paper's n_sync regime: 4 local momentum-SGD steps between exchanges, the sum of the
    # 4 gradients pushed; a step is one cycle (4 minibatches of 32)
    "asgd_nsync4_4x32_bf16": (32, "bf16"),
}
PEAK = {"hbm": 8000.0, "mfma_bf16": 2500.0, "mfma_f32": 157.3}   # GB/s, TFLOP/s (MI355X, dense)
MFMA_CLASSES = ("conv_fwd", "conv_dgrad", "conv_wgrad", "fc_fwd", "fc_dgrad", "fc_wgrad")


STEP_TEXT = {"calls": "fwd_bwd + apply_update_snapshot (push fused with the next fetch)",
             "fused": "train_step_fused (fully-connected weights pushed inside their gradient kernel, the rest in one update launch behind the backward pass)"}


def csrc_hash():
    """Hash of the kernel sources: ties a committed counter summary to the kernels it was measured on."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_1312_6186_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def class_table(prof, K, dtname, hbm_classes=()):
    """Per kernel class: time per step (HIP events around every operation) and the achieved rate on the algorithmic
    work of the class, against the roofline that bounds it.  `hbm_classes`: GEMM classes that are priced against HBM
    (the fully-connected weight gradient once it carries the push: 18 bytes per parameter, two K tiles of MFMAs)."""
    out = {}
    for name, p in prof.items():
        if p["launches"] == 0:
            continue
        ms = p["ms"] / K
        if name in MFMA_CLASSES and name not in hbm_classes:
            ach = p["flops"] / K / (ms * 1e-3) / 1e12
            peak = PEAK["mfma_" + dtname]
            out[name] = {"bound": "mfma", "ms_per_step": ms, "launches_per_step": p["launches"] / K,
                         "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                         "hbm_GBps_on_algorithmic_bytes": p["bytes"] / K / (ms * 1e-3) / 1e9}
        else:
            ach = p["bytes"] / K / (ms * 1e-3) / 1e9
            out[name] = {"bound": "hbm", "ms_per_step": ms, "launches_per_step": p["launches"] / K,
                         "achieved": ach, "peak": PEAK["hbm"], "unit": "GB/s", "frac": ach / PEAK["hbm"]}
    return out


def roofline_of(classes_out, workload):
    """The `roofline` object for the class that takes the most time; HBM bytes per launch from the committed
    rocprofv3 counter summary of this workload, if it was measured on the kernels as they are now."""
    dominant = max(classes_out, key=lambda k: classes_out[k]["ms_per_step"])
    d = classes_out[dominant]
    traffic, note = None, "no counter summary for this workload"
    tpath = os.path.join(ROOT, "profiles", workload + "_hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        t = tj.get("classes", {}).get(dominant)
        if tj.get("csrc_sha256") != csrc_hash():
            note = "the committed counter summary was measured on other kernel sources (%s, now %s)" % (tj.get("csrc_sha256"), csrc_hash())
        elif t:
            traffic = (t["hbm_read_bytes"] + t["hbm_written_bytes"]) / t["launches"]
            note = "profiles/%s_hbm_traffic.json" % workload
    return {"kernel": dominant, "bound": d["bound"], "achieved": d["achieved"], "peak": d["peak"], "unit": d["unit"],
            "frac": d["frac"], "traffic": traffic, "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE)",
            "traffic_source": note,
            "launches_per_step": d["launches_per_step"], "ms_per_launch": d["ms_per_step"] / d["launches_per_step"]}


def cpu_baseline(layers, in_shape, classes, sample_batch, hp):
    """The oracle as it stands, on the host cores: one fwd+bwd+update on `sample_batch` images of the same net."""
    import numpy as np
    import oracle
    from oracle import ops as oops
    from paper_1312_6186_amd import workloads as wl
    net = oracle.OracleNet(layers, in_shape)
    params = wl.make_params(layers, in_shape, 2003).astype(np.float64)
    mom = np.zeros_like(params)
    images, labels = wl.make_batch(in_shape, sample_batch, classes, 1003)
    t0 = time.perf_counter()
    _, grads, _ = net.fwd_bwd(params, images, labels, 3003, 0, 0)
    oops.apply_update(params, mom, grads, hp[0], hp[1], hp[2])
    dt = time.perf_counter() - t0
    return {"value": sample_batch / dt, "unit": "images/sec", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "one fwd+bwd+update of the same AlexNet-style net on %d images (%.1f s)" % (sample_batch, dt)}


def bench_asgd(args, batch, n_sync=0):
    """Replay of a seeded staleness schedule: `steps` pushed gradients, 4 worker streams + a server stream.
    n_sync > 0: the n_sync regime (each push is the sum of n_sync local steps' gradients)."""
    import numpy as np
    import torch
    from paper_1312_6186_amd import binding as B
    from paper_1312_6186_amd import workloads as wl
    cfg = wl.ALEXNET
    layers, in_shape, classes = cfg["layers"], cfg["in_shape"], cfg["classes"]
    lr, mu, wd, W = 1e-3, cfg["mu"], cfg["wd"], 4
    dev = torch.device("cuda:0")
    nets = [B.asgd_net_create(layers, batch, in_shape, B.BF16) for _ in range(W)]
    P = B.asgd_param_count(nets[0])
    params = torch.from_numpy(wl.make_params(layers, in_shape, cfg["seeds"]["init"])).to(dev)
    mom = torch.zeros_like(params)
    copies = [torch.empty(P, dtype=torch.bfloat16, device=dev) for _ in range(W)]
    grads = [torch.empty(P, dtype=torch.float32, device=dev) for _ in range(W)]
    per = max(n_sync, 1)                      # minibatches per pushed gradient
    nb = max(args.steps, args.warmup, 1) * per
    f32 = lambda: [torch.zeros(P, dtype=torch.float32, device=dev) for _ in range(W)]
    wp, wm, wa = (f32(), f32(), f32()) if n_sync else (None, None, None)
    rng = np.random.default_rng(1005)
    images = torch.from_numpy(rng.standard_normal((nb, batch) + tuple(in_shape), dtype=np.float32)).to(dev).to(torch.bfloat16)
    labels = torch.from_numpy(rng.integers(0, classes, size=(nb, batch), dtype=np.int32)).to(dev)
    losses = torch.zeros(nb, dtype=torch.float32, device=dev)
    log = torch.zeros((nb, 3), dtype=torch.int32, device=dev)

    def run(T):
        worker, rv = B.asgd_schedule_generate(T, 4005, W, 3)
        if n_sync:
            B.asgd_replay_nsync_run(nets, n_sync, params, mom, wp, wm, wa, copies, grads, images, labels, worker, rv, lr, mu, wd, 3003,
                                    losses, log)
        else:
            B.asgd_replay_run(nets, params, mom, copies, grads, images, labels, worker, rv, lr, mu, wd, 3003, losses, log)
        torch.cuda.synchronize()
        return worker, rv

    if args.warmup > 0:
        run(args.warmup)
    t0 = time.perf_counter()
    worker, rv = run(args.steps)
    elapsed = time.perf_counter() - t0
    ok = bool((log[:args.steps].cpu().numpy() == np.stack([np.arange(args.steps), worker, rv], 1)).all())
    # Per-class times at the worker shape: the same kernels, one replica alone on one stream with a pair of HIP
    # events around every operation (inside the replay the replicas' kernels overlap and cannot be bracketed).
    stream = torch.cuda.current_stream()
    K = min(args.steps, 8)
    B.asgd_profile_begin(nets[0])
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K)]
    for i in range(K):
        B.asgd_fwd_bwd(nets[0], copies[0], images[i % nb], labels[i % nb], 3003, i, 0, losses[:1], grads[0], stream)
        ev[i][0].record(stream)
        B.asgd_apply_update_snapshot(params, mom, grads[0], lr, mu, wd, copies[0], B.BF16, stream)
        ev[i][1].record(stream)
    torch.cuda.synchronize()
    classes_out = class_table(B.asgd_profile_end(nets[0]), K, "bf16")
    upd_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / K
    classes_out["update_snapshot"] = {"bound": "hbm", "ms_per_step": upd_ms, "launches_per_step": 1, "achieved": P * 22 / (upd_ms * 1e-3) / 1e9,
                                      "peak": PEAK["hbm"], "unit": "GB/s", "frac": P * 22 / (upd_ms * 1e-3) / 1e9 / PEAK["hbm"]}
    for n in nets:
        B.asgd_net_destroy(n)
    cpu = cpu_baseline(layers, in_shape, classes, args.cpu_sample, (lr, mu, wd)) if args.cpu_sample > 0 else None
    print(json.dumps({
        "metric": "images/sec fwd+bwd+update, AlexNet-style bs128; % MFMA peak (conv/FC)",
        "value": batch * per * args.steps / elapsed, "unit": "images/sec", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload,
                   "step": ("one cycle: fetch, %d local steps (fwd_bwd, accumulate, local update) on a worker stream, "
                            "update with the summed gradient on the server stream" % per) if n_sync else
                           "one pushed gradient: snapshot + fwd_bwd on a worker stream, update on the server stream"},
        "workload_detail": {"net": "AlexNet-style single column (%d parameters)" % P, "workers": W, "batch_per_worker": batch,
                            "max_staleness": 3, "schedule_seed": 4005, "n_sync": per, "lr": lr, "mu": mu, "wd": wd},
        "schedule_log_matches": ok,
        "roofline": dict(roofline_of(classes_out, args.workload), measured="one replica alone at the worker shape (batch %d)" % batch),
        "kernel_classes": classes_out, "cpu_baseline": cpu}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="alexnet_bf16_bs128", choices=sorted(WORKLOADS))
    ap.add_argument("--cpu-sample", type=int, default=64, help="images in the oracle's timed sample (0 = skip)")
    ap.add_argument("--serial", action="store_true",
                    help="keep every kernel on one stream (for profiler runs: per-kernel durations are then those of kernels running alone)")
    ap.add_argument("--step", default="fused", choices=["calls", "fused"],
                    help="calls: asgd_fwd_bwd + asgd_apply_update_snapshot; fused: asgd_train_step_fused (the fully-connected "
                         "weights are pushed inside their gradient kernel)")
    args = ap.parse_args()
    if args.serial:
        os.environ["ASGD_SERIAL"] = "1"
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1312_6186_amd import binding as B
    from paper_1312_6186_amd import workloads as wl

    batch, dtname = WORKLOADS[args.workload]
    if args.workload.startswith("asgd_nsync4"):
        return bench_asgd(args, batch, n_sync=4)
    if args.workload.startswith("asgd"):
        return bench_asgd(args, batch)
    dtype = B.BF16 if dtname == "bf16" else B.F32
    tdt = torch.bfloat16 if dtname == "bf16" else torch.float32
    cfg = wl.ALEXNET_FULL if "_full_" in args.workload else wl.ALEXNET_LRN if "_lrn_" in args.workload else wl.ALEXNET
    layers, in_shape, classes = cfg["layers"], cfg["in_shape"], cfg["classes"]
    lr, mu, wd = cfg["lr"], cfg["mu"], cfg["wd"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    net = B.asgd_net_create(layers, batch, in_shape, dtype)
    P = B.asgd_param_count(net)
    master = torch.from_numpy(wl.make_params(layers, in_shape, cfg["seeds"]["init"])).to(dev)
    momentum = torch.zeros_like(master)
    copy = torch.empty(P, dtype=tdt, device=dev)
    grads = torch.empty(P, dtype=torch.float32, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    images_np, labels_np = wl.make_batch(in_shape, batch, classes, cfg["seeds"]["data"])
    images = torch.from_numpy(images_np).to(dev).to(tdt).contiguous()
    labels = torch.from_numpy(labels_np).to(dev)
    B.asgd_net_prepare(net)
    stream = torch.cuda.current_stream()

    # One step of the single-replica loop: the replica's gradient on its copy and the push, which applies the update
    # and leaves the replica's next fetch in `copy`.  "calls": asgd_fwd_bwd, then asgd_apply_update_snapshot over the
    # whole parameter vector.  "fused": asgd_train_step_fused, the same results bit for bit with the fully-connected
    # weights (94 % of the parameters) pushed by the kernel that computes their gradient, which then never goes to
    # memory: 18 instead of 26 bytes of traffic per such parameter.
    fused = args.step == "fused"

    def step(i):
        if fused:
            B.asgd_train_step_fused(net, master, momentum, copy, images, labels, cfg["seeds"]["dropout"], i, 0, loss, grads, lr, mu, wd, stream)
            return
        B.asgd_fwd_bwd(net, copy, images, labels, cfg["seeds"]["dropout"], i, 0, loss, grads, stream)
        B.asgd_apply_update_snapshot(master, momentum, grads, lr, mu, wd, copy, dtype, stream)

    B.asgd_snapshot(master, copy, dtype, stream)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    final_loss = float(loss.item())

    # the same steps again with a pair of HIP events around every operation, on the stream the kernels run on
    B.asgd_profile_begin(net)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    tp0 = time.perf_counter()
    for i in range(args.steps):
        e = ev[i]
        if fused:
            step(args.warmup + args.steps + i)
            continue
        B.asgd_fwd_bwd(net, copy, images, labels, cfg["seeds"]["dropout"], args.warmup + args.steps + i, 0, loss, grads, stream)
        e[0].record(stream)
        B.asgd_apply_update_snapshot(master, momentum, grads, lr, mu, wd, copy, dtype, stream)
        e[1].record(stream)
    torch.cuda.synchronize()
    profiled_ms = 1e3 * (time.perf_counter() - tp0) / args.steps
    prof = B.asgd_profile_end(net)
    # calls that are not part of the step, timed on their own: the two unfused protocol calls and the adaptive updates
    scratch_copy = torch.empty_like(copy)
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(5)]
    zero_grads = torch.zeros_like(grads)
    for e in ev2:
        e[0].record(stream)
        B.asgd_snapshot(master, scratch_copy, dtype, stream)
        e[1].record(stream)
        B.asgd_apply_update(master, momentum, zero_grads, 0.0, 1.0, 0.0, stream)   # lr 0, mu 1: leaves the state as it is
        e[2].record(stream)
    torch.cuda.synchronize()
    K = args.steps
    es = 2 if dtname == "bf16" else 4
    classes_out = class_table(prof, K, dtname, hbm_classes=("fc_wgrad",) if fused else ())
    if not fused:
        upd_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / K
        ach = P * (20 + es) / (upd_ms * 1e-3) / 1e9
        classes_out["update_snapshot"] = {"bound": "hbm", "ms_per_step": upd_ms, "launches_per_step": 1, "achieved": ach, "peak": PEAK["hbm"],
                                          "unit": "GB/s", "frac": ach / PEAK["hbm"]}
    unfused = {}
    for name, a, b, nbytes in (("snapshot", 0, 1, P * (4 + es)), ("update", 1, 2, P * 20)):
        ms = sum(e[a].elapsed_time(e[b]) for e in ev2[1:]) / (len(ev2) - 1)
        unfused[name] = {"bound": "hbm", "ms_per_call": ms, "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK["hbm"], "unit": "GB/s",
                         "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK["hbm"]}
    roofline = roofline_of(classes_out, args.workload)
    # the two adaptive server updates on the same buffers (not part of the step; they leave garbage in `scratch_copy`-sized state)
    state_a, state_b = torch.zeros_like(master), torch.zeros_like(master)
    w_tmp = master.clone()
    ev3 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(5)]
    for e in ev3:
        e[0].record(stream)
        B.asgd_apply_update_adagrad(w_tmp, state_a, zero_grads, 0.01, 1e-7, 5e-4, stream)
        e[1].record(stream)
        B.asgd_apply_update_adadelta(w_tmp, state_a, state_b, zero_grads, 0.95, 1e-6, 5e-4, stream)
        e[2].record(stream)
    torch.cuda.synchronize()
    for name, a, b, nbytes in (("update_adagrad", 0, 1, P * 20), ("update_adadelta", 1, 2, P * 28)):
        ms = sum(e[a].elapsed_time(e[b]) for e in ev3[1:]) / (len(ev3) - 1)
        unfused[name] = {"bound": "hbm", "ms_per_call": ms, "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK["hbm"], "unit": "GB/s",
                         "frac": nbytes / (ms * 1e-3) / 1e9 / PEAK["hbm"]}
    del state_a, state_b, w_tmp
    mfma_names = [n for n, c in classes_out.items() if n in MFMA_CLASSES and c["bound"] == "mfma"]   # (not the GEMM that carries the push)
    mfma_ms = sum(classes_out[n]["ms_per_step"] for n in mfma_names)
    mfma_flops = sum(prof[n]["flops"] for n in mfma_names) / K
    B.asgd_net_destroy(net)

    out = {
        "metric": "images/sec fwd+bwd+update, AlexNet-style bs128; % MFMA peak (conv/FC)",
        "value": batch * args.steps / elapsed, "unit": "images/sec", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtname == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "step": STEP_TEXT[args.step]},
        "workload_detail": {"net": "%s (%d parameters)" % (cfg["name"], P), "batch": batch, "lr": lr, "mu": mu, "wd": wd},
        "loss": final_loss,
        "roofline": roofline,
        "mfma_all_gemms": {"achieved": mfma_flops / (mfma_ms * 1e-3) / 1e12, "peak": PEAK["mfma_" + dtname], "unit": "TFLOP/s",
                           "frac": mfma_flops / (mfma_ms * 1e-3) / 1e12 / PEAK["mfma_" + dtname], "ms_per_step": mfma_ms, "classes": mfma_names},
        "profiled_ms_per_step": profiled_ms, "serial": bool(args.serial),
        "kernel_classes": classes_out,
        "other_calls": unfused,
    }
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(layers, in_shape, classes, args.cpu_sample, (lr, mu, wd))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
