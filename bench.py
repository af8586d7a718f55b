"""Benchmark of the whole training step (forward + pullbacks + SGD-momentum) on one MI355X.

Workload: the ResNet-50-shaped bottleneck net, batch 64 of 3x224x224, bf16 activations and
working weights with fp32 accumulation and fp32 master weights, synthetic N(0,1) inputs.
One "step" is one call of s4tf_train_step over one resident batch.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50] [--no-cpu-baseline]
"""
import argparse
import json
import sys
import time

import numpy as np

METRIC = "train images/sec (fwd+VJP+SGD), ResNet-50 shape bs64 bf16; MFMA util %"
PEAK = {"bf16": 2500.0, "f32": 157.3}   # dense MFMA TFLOP/s, MI355X
HBM_PEAK_TBPS = 8.0

# HBM bytes per launch (reads + writes, averaged over one step's launches of the class) from the hardware
# counters FETCH_SIZE and WRITE_SIZE, each scaled by what it reads for a copy kernel of known size.  The
# figures belong to the kernel sources whose digest is given; with other sources they are not reported.
TRAFFIC = {
    "resnet50": {"sources_sha256": "039dac59fe93c2a7009089ebff66d235b239b4bab38dc55e59a0abcda898e30b",
                 "bytes_per_launch": {"conv_wgrad_igemm": 78.63e6, "conv_dgrad_igemm": 74.38e6, "conv_fwd_igemm": 59.90e6}},
}
TRAFFIC_SOURCES = ("igemm.hip", "igemm_dma.hip", "igemm_args.h", "step.hip")


def measured_traffic(workload, cls):
    import hashlib
    import os
    rec = TRAFFIC.get(workload)
    if not rec or cls not in rec["bytes_per_launch"]:
        return None
    h = hashlib.sha256()
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2102_13243_amd", "csrc")
    for f in TRAFFIC_SOURCES:
        with open(os.path.join(src, f), "rb") as fh:
            h.update(fh.read())
    return rec["bytes_per_launch"][cls] if h.hexdigest() == rec["sources_sha256"] else None


def conv_flops(net, shapes):
    """Algorithmic FLOPs of one step, per kernel class: 2*N*P*Q*K*R*S*C/groups per pass."""
    out = {"conv_fwd_igemm": 0.0, "conv_dgrad_igemm": 0.0, "conv_wgrad_igemm": 0.0,
           "dwconv_fwd": 0.0, "dwconv_dgrad": 0.0, "dwconv_wgrad": 0.0}
    for i, op in enumerate(net["ops"]):
        n, h, w, c = shapes[op["in"]]
        if op["kind"] == "conv":
            _, p, q, k = shapes[i + 1]
            f = 2.0 * n * p * q * k * op["r"] * op["s"] * c / op["groups"]
            pre = "dwconv_" if op["groups"] > 1 else "conv_"
            suf = "" if op["groups"] > 1 else "_igemm"
            out[pre + "fwd" + suf] += f
            out[pre + "wgrad" + suf] += f
            if op["in"] != 0:
                out[pre + "dgrad" + suf] += f
        elif op["kind"] == "head":   # the filter gradient of its dense layer runs on the conv kernel
            out["conv_wgrad_igemm"] += 2.0 * n * c * op["classes"]
    return out


def conv_layerwise_roofline(net, shapes):
    """Per convolution pass, the time the roofline allows it: max(FLOPs / MFMA peak, minimum bytes / HBM peak)
    with the minimum bytes |x| + |w| + |y| at storage width (filter gradient: |x| + |dy| + |dw| in fp32), summed
    over the layers of each class.  Most layers of these nets at their batch sizes are bound by the HBM term."""
    es = 2 if net["dtype"] == "bf16" else 4
    peak = PEAK[net["dtype"]] * 1e12
    out = {"conv_fwd_igemm": 0.0, "conv_dgrad_igemm": 0.0, "conv_wgrad_igemm": 0.0}
    hbm_bound = 0
    layers = 0
    for i, op in enumerate(net["ops"]):
        if op["kind"] != "conv" or op["groups"] > 1:
            continue
        n, h, w, c = shapes[op["in"]]
        _, p, q, k = shapes[i + 1]
        f = 2.0 * n * p * q * k * op["r"] * op["s"] * c
        xb, yb, wn = n * h * w * c * es, n * p * q * k * es, op["r"] * op["s"] * c * k
        layers += 1
        hbm_bound += 1 if (xb + yb + wn * es) / (HBM_PEAK_TBPS * 1e12) > f / peak else 0
        out["conv_fwd_igemm"] += max(f / peak, (xb + yb + wn * es) / (HBM_PEAK_TBPS * 1e12))
        out["conv_wgrad_igemm"] += max(f / peak, (xb + yb + wn * 4) / (HBM_PEAK_TBPS * 1e12))
        if op["in"] != 0:
            out["conv_dgrad_igemm"] += max(f / peak, (xb + yb + wn * es) / (HBM_PEAK_TBPS * 1e12))
    return {k: v * 1e3 for k, v in out.items()}, hbm_bound, layers


def class_bytes(net, shapes, n_params):
    """Algorithmic HBM bytes of one step for the classes that no contraction bounds: every operand a
    kernel class must read or write once, at the storage width (es) of activations; fp32 elsewhere.
      bn_apply       x -> y (+ residual read) (+ activation bits)   (2 + res) * numel * es + bits
      bn_vjp_reduce  x, dy + the activation mask: rebuilt from x      2 * numel * es + mask
                     without a residual (nothing read); with one,
                     the forward pass's bits where the library
                     keeps them (rows of at least 32 bytes of bits
                     per pixel, one bit per element), else y
      bn_vjp_apply   x, dy, mask -> dx (+ residual cotangent, unless  (3 + dres) * numel * es + mask
                     the consuming convolution's dgrad adds it: an
                     identity shortcut in a bf16 net)
      dwconv_fwd     x -> y;  dwconv_dgrad  dy -> dx;  dwconv_wgrad  x, dy      (in + out) * es each
      sgd            p, v, g read, p, v written (fp32) (+ the bf16 working copy written)
    """
    es = 2 if net["dtype"] == "bf16" else 4
    out = {"bn_apply": 0.0, "bn_vjp_reduce": 0.0, "bn_vjp_apply": 0.0, "dwconv_fwd": 0.0, "dwconv_dgrad": 0.0,
           "dwconv_wgrad": 0.0, "sgd": n_params * (20.0 + (2.0 if es == 2 else 0.0))}
    users = {}
    for j, o in enumerate(net["ops"]):
        for t in {o["in"], o.get("res", -1)}:
            if t >= 0:
                users.setdefault(t, []).append(j)
    for i, op in enumerate(net["ops"]):
        numel = float(np.prod(shapes[op["in"]]))
        if op["kind"] == "bn":
            res = 1 if op["res"] >= 0 else 0
            act = 0 if op["act"] == "none" else 1
            c = shapes[op["in"]][3]
            v = 8 if es == 2 else 4
            if c % v:
                v = 1
            bits = numel / v if (res and act and c // v >= 32) else 0.0
            mask = bits if bits else act * res * numel * es
            dres = res
            if bits and es == 2:
                others = [j for j in users.get(op["res"], []) if j != i]
                if len(others) == 1:
                    o = net["ops"][others[0]]
                    if (o["kind"] == "conv" and o["in"] == op["res"] and o["groups"] == 1 and o["stride"] == 1
                            and o["act"] == "none" and shapes[o["in"]][3] % 8 == 0):
                        dres = 0
            out["bn_apply"] += (2 + res) * numel * es + bits
            out["bn_vjp_reduce"] += 2 * numel * es + mask
            out["bn_vjp_apply"] += (3 + dres) * numel * es + mask
        elif op["kind"] == "conv" and op["groups"] > 1:
            io = (numel + float(np.prod(shapes[i + 1]))) * es
            out["dwconv_fwd"] += io
            out["dwconv_dgrad"] += io
            out["dwconv_wgrad"] += io
    return out


def ablation(net, wl, steps, warmup):
    """Eager versus fused (the comparison of the paper's Table 3, on this library's own kernels):
    the same step, same inputs, dispatched three ways.  Each mode gets fresh parameters."""
    import torch
    from paper_2102_13243_amd import binding as B
    from paper_2102_13243_amd.eager import EagerState

    def timed(st):
        xd, ld = st.upload_batch(wl["x"], wl["labels"])
        for _ in range(warmup):
            st.step(xd, ld)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            st.step(xd, ld)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3, float(st.loss[0].item())

    batch = net["input"][0]
    out = {"metric": "train step, fused vs op-by-op dispatch", "workload": net["name"], "batch": batch,
           "dtype": net["dtype"], "steps": steps, "warmup": warmup, "unit": "images/s", "modes": {}}
    for mode, make in (("fused", lambda: B.TrainState(net, wl["params"], "cuda:0")),
                       ("eager_async", lambda: EagerState(net, wl["params"], "cuda:0", sync=False)),
                       ("eager_sync", lambda: EagerState(net, wl["params"], "cuda:0", sync=True))):
        st = make()
        ms, loss = timed(st)
        out["modes"][mode] = {"ms_per_step": round(ms, 4), "images_per_s": round(batch / ms * 1e3, 1),
                              "loss_after": round(loss, 5)}
        del st
        torch.cuda.empty_cache()
    f = out["modes"]["fused"]["ms_per_step"]
    out["fused_speedup_over_eager_sync"] = round(out["modes"]["eager_sync"]["ms_per_step"] / f, 3)
    out["fused_speedup_over_eager_async"] = round(out["modes"]["eager_async"]["ms_per_step"] / f, 3)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other four configurations (other_workloads in the JSON line)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="launch only a plain copy kernel of known size (reads and writes 256 MiB, three times): "
                         "the reference reading for the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--ablation", action="store_true",
                    help="instead of the benchmark line: time the step of --workload three ways, fused "
                         "(s4tf_train_step), op by op with asynchronous dispatch, op by op with a host "
                         "synchronisation after every op (the paper's eager mode), and print one JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_2102_13243_amd import binding as B
    from workloads import nets

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.calibrate_copy:
        n = 64 * 1024 * 1024
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"copy_kernel": "torch.mul(src, 1.0, out=dst)", "bytes_read": 4 * n, "bytes_written": 4 * n, "launches": 3}))
        return
    kw = {"batch": args.batch} if args.batch else {}
    net = nets.CONFIGS[args.workload](**kw)
    wl = nets.make_workload(net)
    if args.ablation:
        print(json.dumps(ablation(net, wl, args.steps, args.warmup)))
        return
    m = measure(net, wl, args.steps, args.warmup, args.workload)
    batch, dtype = net["input"][0], net["dtype"]

    cpu = None
    if not args.no_cpu_baseline:
        # the oracle as it stands on the host's cores, same net, image size and batch as the GPU's step: one
        # warm-up step, one timed step
        cpu = oracle_rate(net, wl, warm=True)
        cpu["sample"] = "one oracle step of the same workload at its full batch %d after one warm-up step (%.1f s)" % (batch, cpu.pop("seconds"))

    others = None
    if args.workload == "resnet50" and not args.no_other_workloads:
        # the other four configurations, short runs: ms per step, images/s, the dominant kernel class against its
        # roofline, and the oracle on the host (all cores; one thread as well for the three small ones)
        others = {}
        for name in ("tiny", "lenet5", "resnet56", "mobilenetv2"):
            onet = nets.CONFIGS[name]()
            owl = nets.make_workload(onet)
            om = measure(onet, owl, 10, 3, name)
            rec = {"ms_per_step": om["ms_per_step"], "images_per_s": om["images_per_s"], "dtype": onet["dtype"],
                   "batch": onet["input"][0], "host_enqueue_ms_per_step": om["host_enqueue_ms_per_step"],
                   "roofline": om["roofline"], "mfma_util_convs": om["mfma_util_convs"]}
            if not args.no_cpu_baseline:
                c = oracle_rate(onet, owl, warm=True)
                rec["cpu_oracle_images_per_s"] = c["value"]
                rec["cpu_cores"] = c["cores"]
                if name != "mobilenetv2":
                    rec["cpu_oracle_images_per_s_1_thread"] = oracle_rate(onet, owl, warm=False, threads=1)["value"]
            others[name] = rec

    out = {
        "metric": METRIC, "value": m["images_per_s"], "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s-shaped net, batch %d of %dx%dx%d, %s storage, fp32 accumulate, SGD-momentum; one "
                               "s4tf_train_step per step" % (net["name"], batch, net["input"][3], net["input"][1],
                                                              net["input"][2], dtype),
                   "params": nets.param_count(wl["params"]), "loss_after": m["loss_after"]},
        "roofline": m["roofline"], "cpu_baseline": cpu,
        "mfma_util_convs": m["mfma_util_convs"],
        "conv_layers_bound_by_hbm": m["conv_layers_bound_by_hbm"],
        "host_enqueue_ms_per_step": m["host_enqueue_ms_per_step"],
        "event_pair_overhead_us": m["event_pair_overhead_us"],
        "kernel_classes": m["kernel_classes"],
        "other_workloads": others,
    }
    print(json.dumps(out))


def oracle_rate(net, wl, warm, threads=None):
    """images/s of one oracle step on the host (optionally after a warm-up step, optionally on `threads` threads)."""
    import os
    import subprocess
    from oracle import oracle as orc
    batch = net["input"][0]
    if threads is not None:
        # the OpenMP thread count is fixed when the oracle's library starts: a child process with its own setting
        code = ("import sys, time, json; sys.path.insert(0, %r); from oracle import oracle as orc; from workloads import nets;"
                "net = nets.CONFIGS[%r](); wl = nets.make_workload(net); t0 = time.perf_counter();"
                "orc.train_step(net, wl['x'], wl['labels'], wl['params']); print(json.dumps([time.perf_counter() - t0, orc.num_threads()]))"
                % (os.path.dirname(os.path.abspath(__file__)), net["name"]))
        env = dict(os.environ, OMP_NUM_THREADS=str(threads))
        ct, cores = json.loads(subprocess.check_output([sys.executable, "-c", code], env=env).decode().strip().splitlines()[-1])
    else:
        if warm:
            orc.train_step(net, wl["x"], wl["labels"], wl["params"])
        t0 = time.perf_counter()
        orc.train_step(net, wl["x"], wl["labels"], wl["params"])
        ct, cores = time.perf_counter() - t0, orc.num_threads()
    return {"value": round(batch / ct, 4), "unit": "images/s", "cores": cores, "kind": "oracle", "seconds": ct}


def measure(net, wl, steps, warmup, workload):
    """Times `steps` training steps of the net on cuda:0 (after `warmup`), then the per-class kernel durations."""
    import torch
    from paper_2102_13243_amd import binding as B
    from workloads import nets
    st = B.TrainState(net, wl["params"], "cuda:0")
    xd, ld = st.upload_batch(wl["x"], wl["labels"])
    batch = net["input"][0]

    for _ in range(warmup):
        st.step(xd, ld)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        st.step(xd, ld)
    t_enq = time.perf_counter() - t0   # the host is done enqueuing; the device is still running
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    loss = float(st.loss[0].item())

    # Per-kernel-class durations: the same steps again with every launch bracketed by HIP events on
    # the launch stream (kept out of the timed region above so the events do not perturb it).
    B.s4tf_profile_enable(True)
    prof_steps = max(1, min(steps, 10))
    for _ in range(prof_steps):
        st.step(xd, ld)
    torch.cuda.synchronize()
    prof = B.s4tf_profile_collect()
    B.s4tf_profile_enable(False)
    # a pair of events also sees the dispatch of the kernel between them; a kernel trace does not
    bracket_ms = max(B.s4tf_profile_bracket_overhead(None, 64), 0.0)
    shapes = nets.tensor_shapes(net)
    flops = conv_flops(net, shapes)
    classes = {}
    for name, (ms, cnt) in prof.items():
        ms = max(ms - cnt * bracket_ms, 0.0)
        classes[name] = {"ms_per_step": ms / prof_steps, "launches_per_step": cnt / prof_steps}
        if flops.get(name) and ms > 0:
            classes[name]["tflops"] = flops[name] / (ms / prof_steps * 1e-3) / 1e12
    nbytes = class_bytes(net, shapes, nets.param_count(wl["params"]))
    for name, b in nbytes.items():
        if b and name in classes and classes[name]["ms_per_step"] > 0:
            classes[name]["hbm_tbps"] = b / (classes[name]["ms_per_step"] * 1e-3) / 1e12
            classes[name]["hbm_frac"] = classes[name]["hbm_tbps"] / HBM_PEAK_TBPS
    dom = max(classes, key=lambda k: classes[k]["ms_per_step"])
    dtype = net["dtype"]
    roofline = None
    if flops.get(dom) and dom.startswith("conv_") and "tflops" in classes[dom]:
        ach = classes[dom]["tflops"]
        roofline = {"bound": "mfma", "kernel": dom, "achieved": round(ach, 2), "peak": PEAK[dtype], "unit": "TFLOP/s",
                    "frac": round(ach / PEAK[dtype], 4), "traffic": measured_traffic(workload, dom),
                    "launches_per_step": classes[dom]["launches_per_step"],
                    "avg_launch_ms": classes[dom]["ms_per_step"] / classes[dom]["launches_per_step"],
                    "flops_per_step": flops[dom]}
    elif "hbm_tbps" in classes[dom]:
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(classes[dom]["hbm_tbps"] * 1e3, 1), "peak": HBM_PEAK_TBPS * 1e3,
                    "unit": "GB/s", "frac": round(classes[dom]["hbm_frac"], 4), "traffic": None,
                    "launches_per_step": classes[dom]["launches_per_step"],
                    "avg_launch_ms": classes[dom]["ms_per_step"] / classes[dom]["launches_per_step"],
                    "bytes_per_step": nbytes[dom]}
    else:   # a class with no roofline model of its own (finalize kernels, pools, the head): time only
        roofline = {"bound": "latency", "kernel": dom, "achieved": None, "peak": None, "unit": None, "frac": None, "traffic": None,
                    "launches_per_step": classes[dom]["launches_per_step"],
                    "avg_launch_ms": classes[dom]["ms_per_step"] / classes[dom]["launches_per_step"]}
    # each convolution class against the sum of its layers' own rooflines (MFMA or HBM, whichever binds the layer)
    roof_ms, hbm_layers, conv_layers = conv_layerwise_roofline(net, shapes)
    for name, ms in roof_ms.items():
        if name in classes and classes[name]["ms_per_step"] > 0 and ms > 0:
            classes[name]["layerwise_roofline_ms"] = ms
            classes[name]["layerwise_roofline_frac"] = ms / classes[name]["ms_per_step"]
    conv_ms = sum(classes[k]["ms_per_step"] for k in ("conv_fwd_igemm", "conv_dgrad_igemm", "conv_wgrad_igemm") if k in classes)
    conv_fl = sum(flops[k] for k in ("conv_fwd_igemm", "conv_dgrad_igemm", "conv_wgrad_igemm"))
    mfma_util = conv_fl / (conv_ms * 1e-3) / 1e12 / PEAK[dtype] if conv_ms else None
    del st
    torch.cuda.empty_cache()
    return {"ms_per_step": round(ms_per_step, 4), "images_per_s": round(batch / (ms_per_step * 1e-3), 1),
            "host_enqueue_ms_per_step": round(t_enq / steps * 1e3, 4), "loss_after": round(loss, 5), "roofline": roofline,
            "mfma_util_convs": None if mfma_util is None else round(mfma_util, 4),
            "conv_layers_bound_by_hbm": "%d of %d" % (hbm_layers, conv_layers),
            "event_pair_overhead_us": round(bracket_ms * 1e3, 3),
            "kernel_classes": {k: {kk: round(vv, 4) for kk, vv in v.items()} for k, v in sorted(classes.items())}}


if __name__ == "__main__":
    main()
