#!/usr/bin/env python3
"""Benchmark of the integer-only inference hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--report FILE]

A "step" is one pass of the whole hot path over one batch of synthetic input.  The default
workload is the one the headline metric is quoted on: the full ResNet50 integer-only forward,
all layers INT8, batch 128 (3x224x224 uint8 images), random seeded folded weights.  Inputs and
weights are resident in HBM before the timed region.  Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5033.0     # MI355X dense INT8 MFMA, published (5.0 POP/s)
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published

# Transition blocks (the first block of every stage) of the all-INT8 workloads run in the form of the paper's Figure 2: the
# block's last convolution and the transition convolution both stay INT32 and are rescaled and added in one launch.  The
# "_stored" variants keep the transition convolution's output as a signed 8-bit tensor value first (same launches wherever
# the pair can be fused, one more rounding); the networks with 4-bit layers use that form throughout.
WORKLOADS = {
    "resnet50_int8_b128": dict(arch=50, batch=128, mixed=False, seed=1003, int32_shortcut=True),
    "resnet18_int8_b64": dict(arch=18, batch=64, mixed=False, seed=1002, int32_shortcut=True),
    "resnet50_mixed_b256": dict(arch=50, batch=256, mixed=True, seed=1004),
    "resnet50_int4_b128": dict(arch=50, batch=128, mixed="all4", seed=1005),
    "resnet50_int8_b128_stored": dict(arch=50, batch=128, mixed=False, seed=1003),
    "resnet50_int8_b256_stored": dict(arch=50, batch=256, mixed=False, seed=1004),   # the all-INT8 twin of resnet50_mixed_b256
    "resnet50_int4_b256": dict(arch=50, batch=256, mixed="all4", seed=1004),
    "resnet18_int8_b64_stored": dict(arch=18, batch=64, mixed=False, seed=1002),
}


def cpu_baseline(net, images):
    """Time the CPU oracle (as it stands) on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    from oracle import resnet as onet
    import workloads as wl
    oracle.lib()
    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    x = wl.make_image_batch(99, images, image_hw=net["image_hw"])
    onet.forward(net, x[:1])  # page in
    t0 = time.perf_counter()
    onet.forward(net, x)
    dt = time.perf_counter() - t0
    return dict(value=images / dt, unit="images/s", cores=cores, kind="oracle",
                sample="%d images of the same network and input distribution, %.1f s" % (images, dt),
                build="gcc " + " ".join(oracle.CFLAGS) + " (plain C loops, OpenMP over output pixels, no intrinsics, no BLAS)")


def _profile_text(workload):
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "forward_%s.md" % workload)
    try:
        return open(path).read()
    except OSError:
        return None


def profiled_traffic(workload):
    """HBM bytes one forward moved under rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel
    calibration), read from the committed summary of that profile; None if there is none for this workload."""
    text = _profile_text(workload)
    if text is None:
        return None
    m = re.search(r"all kernels of one forward, scaled by the copy factors: read ([0-9.]+) MB, written ([0-9.]+) MB", text)
    return (float(m.group(1)) + float(m.group(2))) * 1e6 if m else None


def profiled_dominant_kernel(workload):
    """The kernel with the largest share of a forward in the committed rocprofv3 summary (one-stream run, kernel-trace
    durations and counters): name, launches and microseconds per forward, its HBM and INT8-MFMA rates against the
    published peaks and which of the two it is nearer to; None if there is no summary for this workload."""
    text = _profile_text(workload)
    if text is None or "## Derived per kernel" not in text:
        return None
    best = None
    for line in text.split("## Derived per kernel", 1)[1].splitlines():
        c = [x.strip() for x in line.strip().strip("|").split("|")]
        if len(c) != 9 or not c[1].isdigit():
            continue
        row = dict(name=c[0].strip("`"), launches_per_forward=int(c[1]), us_per_forward=float(c[2]), hbm_mb=float(c[3]),
                   hbm_gbs=float(c[4]), frac_hbm_peak=float(c[5]), tops=float(c[6]), frac_int8_mfma_peak=float(c[7]),
                   mfma_pipe_busy=float(c[8]))
        if best is None or row["us_per_forward"] > best["us_per_forward"]:
            best = row
    if best is not None:
        best["bound"] = "mfma" if best["frac_int8_mfma_peak"] >= best["frac_hbm_peak"] else "hbm"
        best["frac"] = max(best["frac_int8_mfma_peak"], best["frac_hbm_peak"])
        best["source"] = "profiles/forward_%s.md" % workload
    return best


def dominant_kernel_layers(workload, kernel):
    """Names of the layers that the committed launch-by-launch summary (profiles/per_layer_<workload>.md) shows on `kernel`."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "per_layer_%s.md" % workload)
    if not os.path.exists(path):
        return []
    names = []
    for line in open(path):
        c = [x.strip() for x in line.strip().strip("|").split("|")]
        if len(c) >= 5 and c[0].isdigit() and c[3].strip("`") == kernel:
            names.append(c[1])
    return names


def conv_sweep(hawq, torch, wl, np):
    """Single-layer configurations: the 56x56x64 3x3 layer (batch 1 as specified, batch 128 as a throughput companion) and
    the ResNet18-shaped 3x3 / strided / 1x1 sweep in INT4 and in INT8 (batch 8 as specified, and batch 128), seeded inputs
    resident in HBM (weights as given and as the blocked copy of hawq_conv_block_weights), median of 20 HIP-event timed
    launches after 5 warm-ups.  TOPS = 2 N P Q K R S C / t (logical MACs)."""
    def run(N, H, W, C, K, R, S, stride, pad, bits, seed):
        case = wl.conv_case(seed=seed, N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride=stride, pad=pad, bits=bits)
        x_dt, w_dt = (hawq.U8, hawq.S8) if bits == 8 else (hawq.U4, hawq.S4)
        P, Q = case["P"], case["Q"]
        d = hawq.ConvDesc(N=N, H=H, W=W, C=C, K=K, R=R, S=S, stride_h=stride, stride_w=stride, pad_h=pad, pad_w=pad, x_dtype=x_dt,
                          w_dtype=w_dt, y_dtype=x_dt, res_dtype=hawq.U8, relu=1, y_lo=0, y_hi=127 if bits == 8 else 15,
                          x_hi=127 if bits == 8 else 0)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        x, w, bias, b, c = dev(case["x"]), dev(case["w"]), dev(case["bias"]), dev(case["b"]), dev(case["c"])
        y = torch.empty((N, P, Q, K if bits == 8 else K // 2), dtype=torch.uint8, device="cuda")
        nb = hawq.hawq_conv_blocked_weights_bytes(d)     # the weights also in the blocked order, made once outside the timing
        if nb:
            wb = torch.empty(nb, dtype=torch.uint8, device="cuda")
            hawq.hawq_conv_block_weights(d, w, wb)
            d.w_blocked = wb.data_ptr()
        nf = hawq.hawq_conv_fragment_weights_bytes(d)    # ... and in matrix-instruction fragment order (resident-pixel kernel)
        if nf and R == 3 and stride == 1:
            wf = torch.empty(nf, dtype=torch.uint8, device="cuda")
            hawq.hawq_conv_fragment_weights(d, w, wf)
            d.w_fragments = wf.data_ptr()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for _ in range(5):
            hawq.hawq_conv2d_int(d, x, w, bias, b, c, None, None, None, y)
        for e0, e1 in ev:
            e0.record()
            hawq.hawq_conv2d_int(d, x, w, bias, b, c, None, None, None, y)
            e1.record()
        torch.cuda.synchronize()
        us = float(np.median([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e3
        ops = 2.0 * N * P * Q * K * R * S * C
        return dict(N=N, H=H, W=W, C=C, K=K, R=R, stride=stride, bits=bits, us=round(us, 2), tops=round(ops / us / 1e6, 1),
                    frac_mfma_peak=round(ops / us / 1e6 / PEAK_INT8_TOPS, 4))
    rows = []
    for N in (1, 128):
        rows.append(dict(config="single 3x3 layer", **run(N, 56, 56, 64, 64, 3, 3, 1, 1, 8, 1000)))
    for batch in (8, 128):
        for name, N, H, W, C, K, R, S, stride, pad in wl.int4_sweep_shapes(batch):
            for bits in (4, 8):
                rows.append(dict(config="sweep " + name, **run(N, H, W, C, K, R, S, stride, pad, bits, 1001)))
    loop_peak = hawq.hawq_probe_mfma_peak(20000)   # TOP/s of a register-only INT8 MFMA loop on this device (now warm)
    for r in rows:
        r["frac_mfma_loop_peak"] = round(r["tops"] / loop_peak, 4)
    return {"workload": "single-layer configurations (event-timed launches include ~2 us of launch overhead)",
            "mfma_peak_tops": PEAK_INT8_TOPS, "mfma_loop_peak_tops": round(loop_peak, 1), "rows": rows}


def module_ops(hawq, torch, steps, warmup):
    """Algorithmic GB/s of hawq_pool2d_sum_int and hawq_concat_dyadic at the size of an Inception 35x35 module, batch 128
    (synthetic INT32 feature maps resident in HBM; HIP events on the launch stream)."""
    N, H, Ks = 128, 35, (64, 64, 96, 64)
    P, C = N * H * H, sum(Ks)
    g = torch.Generator(device="cuda").manual_seed(7)
    qs = [torch.randint(-(1 << 20), 1 << 20, (P, K), dtype=torch.int32, device="cuda", generator=g) for K in Ks]
    bs = [torch.randint(1 << 14, 1 << 15, (K,), dtype=torch.int32, device="cuda", generator=g) for K in Ks]
    cs = [torch.full((K,), 28, dtype=torch.uint8, device="cuda") for K in Ks]
    y = torch.empty((P, C), dtype=torch.uint8, device="cuda")
    br = [(q, hawq.S32, b, c) for q, b, c in zip(qs, bs, cs)]
    x = torch.randint(0, 1 << 20, (N, H, H, C), dtype=torch.int32, device="cuda", generator=g)
    yp = torch.empty((N, H, H, C), dtype=torch.int32, device="cuda")

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps
    t_cat = timed(lambda: hawq.hawq_concat_dyadic(P, br, hawq.U8, 0, 127, y))
    t_pool = timed(lambda: hawq.hawq_pool2d_sum_int(N, H, H, C, 3, 3, 1, 1, 1, 1, hawq.S32, hawq.S32, x, None, None, 0, 0, yp))
    return {"workload": "inception 35x35 module operators, batch 128, %d channels" % C,
            "concat_dyadic": {"us": t_cat * 1e3, "algorithmic_bytes": P * C * 5, "GBps": P * C * 5 / t_cat / 1e6, "frac_hbm_peak": P * C * 5 / t_cat / 1e6 / PEAK_HBM_GBS},
            "pool2d_sum_int32": {"us": t_pool * 1e3, "algorithmic_bytes": P * C * 8, "GBps": P * C * 8 / t_pool / 1e6, "frac_hbm_peak": P * C * 8 / t_pool / 1e6 / PEAK_HBM_GBS}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (a forward is ~1 ms: a few dozen steps end before clocks and caches have settled and read ~3 % low)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="resnet50_int8_b128", choices=sorted(WORKLOADS))
    ap.add_argument("--cpu-images", type=int, default=256, help="images in the CPU-oracle baseline sample (0: skip)")
    ap.add_argument("--report", default=None, help="optional file for the per-layer table (JSON)")
    ap.add_argument("--bits-json", default=None,
                    help="JSON file {group name: 4 | 8} replacing the workload's bit assignment (e.g. a selection written by "
                         "`python -m paper_2011_10680_amd.bitselect_report`)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy kernel 5 times (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--single-stream", action="store_true",
                    help="run the batch as one part on one stream (the library otherwise runs a batch of 96 or more as two "
                         "halves on two streams); for per-kernel profiles, where overlapping kernels blur the durations")
    ap.add_argument("--split", type=int, default=0,
                    help="run the batch as two parts on two streams with this many images in the first part (0: the library's rule)")
    ap.add_argument("--fuse-tails", type=int, default=0,
                    help="1: run the 3x3 -> 1x1 + shortcut tails of identity bottleneck blocks as one launch wherever the fused "
                         "kernel applies; 2: only the 256-channel blocks (measurement of hawq_bottleneck_tail_int inside the network; "
                         "0: the plan's rule)")
    ap.add_argument("--conv-sweep", action="store_true",
                    help="time the single-layer configurations (one 3x3 layer; the ResNet18-shaped INT4 / INT8 sweep) and exit")
    ap.add_argument("--module-ops", action="store_true",
                    help="time the two memory-bound operators of an Inception-style module instead (INT32 3x3 window-sum "
                         "pool and the concatenation with one dyadic number per branch, 128 x 35 x 35 x 288) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (images are independent: more GPUs would each take a share of "
              "the batch, with no exchange) -- run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    if args.copy_calibration:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 1 << 30, "copy_calibration_bytes_written": 1 << 30, "launches": 5}))
        return
    import workloads as wl
    import paper_2011_10680_amd as hawq

    hawq.load_library()   # fails loudly if libhawq.so is not built: there is no fallback path
    if args.conv_sweep:
        print(json.dumps(conv_sweep(hawq, torch, wl, np)))
        return
    if args.module_ops:
        print(json.dumps(module_ops(hawq, torch, args.steps, args.warmup)))
        return
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wk = WORKLOADS[args.workload]
    arch, N = wk["arch"], wk["batch"]
    if wk["mixed"] == "all4":
        bits = {g: (8 if g in ("conv1", "fc") else 4) for g in wl.resnet_group_names(arch)}
    elif wk["mixed"]:
        bits = wl.draw_bits(arch, 4000 + arch)
    else:
        bits = None
    if args.bits_json:
        with open(args.bits_json) as f:
            bits = {k: int(v) for k, v in json.load(f).items()}
    net = wl.make_resnet(arch, seed=wk["seed"], bits=bits, int32_shortcut=wk.get("int32_shortcut", False) and not args.bits_json)
    x = torch.from_numpy(wl.make_image_batch(wk["seed"] + 1, N)).cuda()
    hawq.hawq_tune_set_fusion(args.fuse_tails)
    hn = hawq.HawqNet(arch, net["layers"], net["pool_b"], net["pool_c"])
    hawq.hawq_tune_set_fusion(0)
    if args.single_stream:
        hawq.hawq_tune_set_split(-1)
    elif args.split > 0:
        hawq.hawq_tune_set_split(args.split)
    first = hn.split_first(N)
    ws = torch.empty(hn.workspace_bytes(N), dtype=torch.uint8, device="cuda")
    logits = torch.empty((N, 1000), dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    for _ in range(args.warmup):
        hn.hawq_forward_resnet(x, N, logits, ws, stream)
    torch.cuda.synchronize()
    # the K timed steps, bracketed by synchronisation (wall clock) and by two HIP events recorded on the
    # stream the library launches on (device time of the whole region)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        hn.hawq_forward_resnet(x, N, logits, ws, stream)
    ev1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_ms_per_step = ev0.elapsed_time(ev1) / args.steps

    loop_peak = hawq.hawq_probe_mfma_peak(20000)
    # per-launch device times (HIP events recorded by the library on the same stream), median of a few passes
    reps = max(3, min(10, args.steps))
    per = np.array([hn.hawq_forward_resnet_timed(x, N, logits, ws, stream) for _ in range(reps)])
    step_ms = np.median(per, axis=0)
    nsteps = hn.num_steps()
    rows = []
    for s in range(nsteps):
        macs, nbytes = hn.step_cost(N, s)
        o = hn.step_output(N, s)
        rows.append(dict(step=s, name=o["name"], dims="%d,%d,%d,%d" % o["dims"], ms=float(step_ms[s]), gmac=macs / 1e9, mbytes=nbytes / 1e6,
                         tops=2 * macs / (step_ms[s] * 1e-3) / 1e12 if macs else 0.0,
                         gbs=nbytes / (step_ms[s] * 1e-3) / 1e9))
    total_macs = sum(r["gmac"] for r in rows) * 1e9
    conv_rows = [r for r in rows if r["gmac"] > 0 and r["name"] not in ("conv1", "fc")]
    conv_ms = sum(r["ms"] for r in conv_rows)
    conv_bytes = sum(r["mbytes"] for r in conv_rows) * 1e6
    conv_ops = 2 * sum(r["gmac"] for r in conv_rows) * 1e9
    # Roofline of the path.  One "launch" is one forward: the chain of kernels (fused conv1 + max pool, the
    # matrix-core convolutions, average pool, FC) over one batch.  Algorithmic bytes: every layer reads its
    # input (and shortcut) once and writes its output once, weights and per-channel parameters once.  At
    # 8 TB/s those bytes take longer than the forward's MACs at the INT8 MFMA peak, so the bound is HBM.
    # Duration: the two HIP events around the timed region, per step.
    total_bytes = sum(r["mbytes"] for r in rows) * 1e6
    total_ops = 2 * total_macs
    t_mem = total_bytes / (PEAK_HBM_GBS * 1e9)
    t_mfma = total_ops / (PEAK_INT8_TOPS * 1e12)
    achieved_gbs = total_bytes / (ev_ms_per_step * 1e-3) / 1e9
    achieved_tops = total_ops / (ev_ms_per_step * 1e-3) / 1e12
    if t_mem >= t_mfma:
        roof = dict(bound="hbm", achieved=achieved_gbs, peak=PEAK_HBM_GBS, unit="GB/s", frac=achieved_gbs / PEAK_HBM_GBS)
    else:
        roof = dict(bound="mfma", achieved=achieved_tops, peak=PEAK_INT8_TOPS, unit="TOP/s", frac=achieved_tops / PEAK_INT8_TOPS)
    # the profile's dominant kernel, cross-checked live: this run's per-launch event times (one stream; each interval holds
    # a few microseconds of launch and event overhead) of the layers the committed launch-by-launch summary shows on it
    dom = profiled_dominant_kernel(args.workload)
    if dom is not None and not args.bits_json:
        layers = set(dominant_kernel_layers(args.workload, dom["name"]))
        live = [r for r in rows if r["name"] in layers]
        if live and len(live) == dom["launches_per_forward"]:
            live_us = sum(r["ms"] for r in live) * 1e3
            dom["live_event_us_per_forward"] = live_us
            dom["live_tops"] = 2 * sum(r["gmac"] for r in live) * 1e9 / (live_us * 1e-6) / 1e12
            dom["live_frac_int8_mfma_peak"] = dom["live_tops"] / PEAK_INT8_TOPS
    roof.update(traffic=profiled_traffic(args.workload),
                kernel="one forward = %s%d launches (conv_stem_pool, conv3x3_c64, conv_rp, conv_mfma, conv_pw, conv_pws, conv_pws_dual, avgpool)"
                       % ("2 x " if first else "", sum(r["mbytes"] > 0 for r in rows)),
                dominant_kernel=dom,
                launch_ms=ev_ms_per_step, algorithmic_bytes=total_bytes, t_hbm_ms=t_mem * 1e3, t_mfma_ms=t_mfma * 1e3,
                mfma_tops=achieved_tops, mfma_frac=achieved_tops / PEAK_INT8_TOPS,
                # the same against what a register-only INT8 MFMA loop sustains on this device, measured now
                mfma_loop_peak_tops=loop_peak, mfma_frac_of_loop_peak=achieved_tops / loop_peak,
                # the matrix-core convolutions alone, from per-launch events (each interval also holds a few
                # microseconds of launch and event overhead that the untimed forward does not pay)
                conv_kernels=dict(launches=len(conv_rows), launches_ms=conv_ms, gbs=conv_bytes / (conv_ms * 1e-3) / 1e9,
                                  tops=conv_ops / (conv_ms * 1e-3) / 1e12))

    out = {
        "metric": "resnet%d_int_only_images_per_sec" % arch, "value": N / (ms_per_step * 1e-3), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8" if not any(l["bits"] == 4 for l in net["layers"]) else "int4/int8", "data": "synthetic",
        "config": {"workload": args.workload + (" with --bits-json" if args.bits_json else ""), "batch": N, "image": "3x224x224 uint8",
                   "layers_int4": sum(l["bits"] == 4 for l in net["layers"]),
                   "transition_blocks": "int32 both branches" if (wk.get("int32_shortcut") and not args.bits_json) else "stored int8 shortcut",
                   "batch_parts": "%d + %d images on two streams" % (first, N - first) if first else "one"},
        "tops": 2 * total_macs / (ms_per_step * 1e-3) / 1e12,
        "frac_int8_mfma_peak": 2 * total_macs / (ms_per_step * 1e-3) / 1e12 / PEAK_INT8_TOPS,
        "sum_kernel_ms": float(step_ms.sum()),
        "roofline": roof,
    }
    if args.cpu_images > 0:
        out["cpu_baseline"] = cpu_baseline(net, args.cpu_images)
    if args.report:
        os.makedirs(os.path.dirname(os.path.abspath(args.report)), exist_ok=True)
        with open(args.report, "w") as f:
            json.dump(dict(summary=out, layers=rows), f, indent=1)
    hn.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
