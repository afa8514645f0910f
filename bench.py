#!/usr/bin/env python3
"""Benchmark: labelled pixels/s of whole-image forward + backward on one MI355X.

A step is one pass of the whole hot path over one synthetic batch that is already
resident in HBM: pad -> every sparse-kernel conv / pool layer -> masked softmax
cross-entropy -> error maps and all weight / bias gradients.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--dtype f32|bf16]
                  [--forward-only] [--no-cpu-baseline] [--algo 0|1]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA = 157.3      # TFLOP/s, MI355X dense fp32 matrix
PEAK_BF16_MFMA = 2500.0     # TFLOP/s, MI355X dense bf16 matrix
PEAK_HBM = 8000.0           # GB/s
kDenseIntensity = 100.0     # flop per byte from which a conv layer counts as a dense contraction
# The paper's own measurement of configs[5] (Plain CNN_1, 3x388x388 padded, Tesla K40, fp32; Table 1):
# forward 35.39 ms, backward 91.26 ms for 256 x 256 labelled pixels.  Another machine: context, not a target.
PAPER_PLAIN_CNN1_MS = {"fwd": 35.39, "fwd+bwd": 35.39 + 91.26}


def warm_event_pool(torch, count):
    """The per-call events of the timed region are instrumentation, not part of the path: the HIP runtime grows its
    event pool in large steps (one of them stalls the host for tens of milliseconds near the thousandth live event),
    which a launch-bound workload would see as a slow step.  Creating and recording that many events once, before
    the clock starts, leaves the pool grown."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(count)]
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    del ev


def layer_costs(net, elem):
    """Algorithmic work per library call: FLOPs of the non-zero taps for convs,
    minimum bytes (each input element read once, each output written once) for the rest."""
    import paper_1412_4526_amd as dsk
    N, out = net.N, {}
    L = len(net.plan)
    for l, p in enumerate(net.plan):
        nin, nout = N * p.C * p.H * p.W, N * p.K * p.Ho * p.Wo
        oel = 4 if l == L - 1 else elem
        if p.kind == dsk.DSK_CONV:
            fl = 2.0 * N * p.C * p.K * p.k * p.k * p.Ho * p.Wo
            wb = p.K * p.C * p.k * p.k * 4
            out[("conv_fwd", l)] = dict(flops=fl, bytes=nin * elem + nout * oel + wb)
            out[("conv_bwd_data", l)] = dict(flops=fl, bytes=nout * oel + nin * elem + wb)
            out[("conv_bwd_weight", l)] = dict(flops=fl, bytes=nin * elem + nout * oel + wb)
            # backward-data with the non-linearity backward of the conv layer below: that layer's output is read too
            out[("conv_bwd_data_act", l)] = dict(flops=fl, bytes=nout * oel + 2 * nin * elem + wb)
            out[("act_bwd", l)] = dict(flops=0.0, bytes=3 * nout * oel)
        elif p.kind == dsk.DSK_MAXPOOL:
            out[("maxpool_fwd", l)] = dict(flops=0.0, bytes=nin * elem + nout * (elem + 1))
            out[("maxpool_bwd", l)] = dict(flops=0.0, bytes=nout * (elem + 1) + nin * elem)
            # fused with the non-linearity backward of the conv layer in front: that layer's output is read too
            out[("pool_bwd_act", l)] = dict(flops=0.0, bytes=nout * (elem + 1) + 2 * nin * elem)
        else:
            out[("avgpool_fwd", l)] = dict(flops=0.0, bytes=nin * elem + nout * elem)
            out[("avgpool_bwd", l)] = dict(flops=0.0, bytes=nout * elem + nin * elem)
            out[("pool_bwd_act", l)] = dict(flops=0.0, bytes=nout * elem + 2 * nin * elem)
    last = net.plan[-1]
    px = N * last.Ho * last.Wo
    out[("softmax_xent", L)] = dict(flops=0.0, bytes=px * (last.K * 4 + 4 + 1 + last.K * elem))
    out[("pad", -1)] = dict(flops=0.0, bytes=N * net.net.C0 * (net.H * net.W * 4 + net.maps[0].shape[2] * net.maps[0].shape[3] * elem))
    return out


def cpu_baseline(cfg, wl, forward_only, budget_s=20.0):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of
    the same workload: patches are independent and equal-cost, so px/s = patches/s."""
    import numpy as np
    import oracle
    from workloads import sample_pixels
    net = cfg.net
    params = oracle.pack_params(wl.weights, wl.biases)
    xpad = oracle.pad_image(wl.image, net.patch)
    threads = oracle.num_threads()
    N, _, H, W = wl.image.shape
    probe = sample_pixels(N, H, W, threads, seed=11)

    def run(pix):
        t0 = time.perf_counter()
        s = oracle.scan_forward(net, params, xpad, pix)
        if not forward_only:
            d = np.full((len(pix), net.classes), 1.0 / len(pix))
            oracle.scan_backward(net, params, xpad, pix, d)
        return time.perf_counter() - t0

    t_probe = run(probe)
    count = int(max(threads, min(N * H * W, threads * max(1.0, budget_s / max(t_probe, 1e-3)))))
    count -= count % threads
    pix = sample_pixels(N, H, W, count, seed=12)
    t = run(pix)
    return {"value": len(pix) / t, "unit": "labelled pixels/s", "cores": threads, "kind": "oracle",
            "sample": "%d patches of %dx%d (of %d pixels), %s, patch-by-patch fp64, %.1f s"
                      % (len(pix), net.patch, net.patch, N * H * W,
                         "forward only" if forward_only else "forward + backward", t)}


def video_costs(net, elem):
    """Algorithmic work per library call of a video network (3-D layers): FLOPs of the non-zero taps for convs,
    minimum bytes for the rest."""
    import paper_1412_4526_amd as dsk
    N, out = net.N, {}
    L = len(net.plan)
    for l, (p, q) in enumerate(zip(net.plan, net.tplan)):
        nin, nout = N * q.H * p.C * p.H * p.W, N * q.Ho * p.K * p.Ho * p.Wo
        oel = 4 if l == L - 1 else elem
        if p.kind == dsk.DSK_CONV:
            fl = 2.0 * N * q.Ho * p.C * p.K * q.k * p.k * p.k * p.Ho * p.Wo
            wb = q.k * p.K * p.C * p.k * p.k * 4
            for tag in ("conv3d_fwd", "conv3d_bwd_data", "conv3d_bwd_weight"):
                out[(tag, l)] = dict(flops=fl, bytes=nin * elem + nout * oel + wb)
            out[("act_bwd", l)] = dict(flops=0.0, bytes=3 * nout * oel)
            out[("conv_bwd_data_act", l)] = dict(flops=fl, bytes=nout * oel + 2 * nin * elem + wb)
        elif p.kind == dsk.DSK_MAXPOOL:
            out[("maxpool3d_fwd", l)] = dict(flops=0.0, bytes=nin * elem + nout * (elem + 1))
            out[("maxpool3d_bwd", l)] = dict(flops=0.0, bytes=nout * (elem + 1) + nin * elem)
        else:
            out[("avgpool3d_fwd", l)] = dict(flops=0.0, bytes=nin * elem + nout * elem)
            out[("avgpool3d_bwd", l)] = dict(flops=0.0, bytes=nout * elem + nin * elem)
    last = net.plan[-1]
    vox = N * net.T * net.H * net.W
    out[("softmax_xent", L)] = dict(flops=0.0, bytes=vox * (last.K * 4 + 4 + 1 + last.K * elem))
    out[("pad", -1)] = dict(flops=0.0, bytes=N * net.T * net.net.C0 * net.H * net.W * 4 + net.xpad.numel() * elem)
    return out


def video_cpu_baseline(cfg, wl, forward_only, budget_s=20.0):
    """The cube-scanning oracle on this machine's host cores, on a bounded sample of the clip's voxels."""
    import numpy as np
    import oracle
    net = cfg.net
    params = oracle.pack_params3d(wl.weights, wl.biases)
    xpad = oracle.pad_video(wl.video, net.patch_t, net.patch)
    threads = oracle.num_threads()
    rng = np.random.default_rng(11)

    def sample(count):
        return np.stack([rng.integers(0, cfg.N, count), rng.integers(0, cfg.T, count), rng.integers(0, cfg.H, count),
                         rng.integers(0, cfg.W, count)], 1).astype(np.int32)

    def run(vox):
        t0 = time.perf_counter()
        oracle.cube_scan_forward(net, params, xpad, vox)
        if not forward_only:
            oracle.cube_scan_backward(net, params, xpad, vox, np.full((len(vox), net.classes), 1.0 / len(vox)))
        return time.perf_counter() - t0

    t_probe = run(sample(threads))
    count = int(max(threads, threads * max(1.0, budget_s / max(t_probe, 1e-3))))
    count -= count % threads
    vox = sample(count)
    t = run(vox)
    return {"value": len(vox) / t, "unit": "labelled voxels/s", "cores": threads, "kind": "oracle",
            "sample": "%d cubes of %dx%dx%d (of %d voxels), %s, cube-by-cube fp64, %.1f s"
                      % (len(vox), net.patch_t, net.patch, net.patch, cfg.N * cfg.T * cfg.H * cfg.W,
                         "forward only" if forward_only else "forward + backward", t)}


def main_video(args):
    """--video I: the same measurement on a video workload (3-D convolution and pooling; Sec. 6)."""
    import numpy as np
    import torch
    import paper_1412_4526_amd as dsk
    from workloads import VIDEO_CONFIGS, make_video_workload

    cfg = VIDEO_CONFIGS[args.video]
    dtype = args.dtype or cfg.dtype
    elem = 4 if dtype == "f32" else 2
    wl = make_video_workload(cfg.net, cfg.N, cfg.T, cfg.H, cfg.W, cfg.mask_frac, cfg.seed)
    dev = "cuda:0"
    dsk.dsk_set_conv_algo(args.algo)
    net = dsk.WholeVideoNet(cfg.net, cfg.N, cfg.T, cfg.H, cfg.W, dtype, dev, train=not args.forward_only)
    net.load_params(wl.weights, wl.biases)
    video = torch.from_numpy(np.ascontiguousarray(np.transpose(wl.video, (0, 2, 1, 3, 4)))).to(dev)
    labels = torch.from_numpy(wl.labels).to(dev)
    mask = torch.from_numpy(wl.mask).to(dev)

    def step():
        net.forward(video)
        if not args.forward_only:
            net.loss_backward(labels, mask)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    warm_event_pool(torch, 8192 + 2 * (2 * len(net.plan) + 4) * args.steps)
    net.timeline = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    timeline, net.timeline = net.timeline, None
    per = {}
    for tag, layer, e0, e1 in timeline:
        per.setdefault((tag, layer), []).append(e0.elapsed_time(e1))
    costs = video_costs(net, elem)
    rows = []
    for key, ms in per.items():
        avg = sum(ms) / len(ms)
        c = costs[key]
        row = {"call": key[0], "layer": key[1], "ms": round(avg, 4)}
        if 0 <= key[1] < len(net.plan):
            p, q = net.plan[key[1]], net.tplan[key[1]]
            row["shape"] = "C%d K%d kt%d k%d dt%d d%d %dx%dx%d" % (p.C, p.K, q.k, p.k, q.d, p.d, q.H, p.H, p.W)
        if c["flops"] > 0:
            row["tflops"] = round(c["flops"] / avg / 1e9, 2)
            row["intensity"] = round(c["flops"] / c["bytes"], 1)
        row["gbs"] = round(c["bytes"] / avg / 1e6, 1)
        rows.append(row)
    if args.layers:
        for r in sorted(rows, key=lambda r: -r["ms"]):
            sys.stderr.write(json.dumps(r) + "\n")
    dom = max(rows, key=lambda r: r["ms"])
    c = costs[(dom["call"], dom["layer"])]
    peak_mfma = PEAK_FP32_MFMA      # video layers run on the fp32 matrix cores in both storage types
    if c["flops"] > 0 and c["flops"] / c["bytes"] >= peak_mfma * 1e3 / PEAK_HBM:
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": peak_mfma, "unit": "TFLOP/s",
                "frac": round(dom["tflops"] / peak_mfma, 4)}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": PEAK_HBM, "unit": "GB/s", "frac": round(dom["gbs"] / PEAK_HBM, 4)}
    roof.update(traffic=None, algorithmic_bytes=int(c["bytes"]), algorithmic_flops=int(c["flops"]),
                kernel="%s layer %d (%s)" % (dom["call"], dom["layer"], dom.get("shape", "")), ms=dom["ms"])
    voxels = cfg.N * cfg.T * cfg.H * cfg.W
    worst_conv = min((r["tflops"] / peak_mfma for r in rows if "tflops" in r and r["intensity"] >= kDenseIntensity), default=None)
    worst_pool = min((r["gbs"] / PEAK_HBM for r in rows if "pool" in r["call"]), default=None)
    out = {
        "metric": "labelled voxels/s whole-video %s" % ("fwd" if args.forward_only else "fwd+bwd"),
        "value": voxels * args.steps / dt, "unit": "labelled voxels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "video[%d]: %s cube %dx%dx%d, %dx%dx%dx%dx%d clip, mask %.0f%%"
                               % (args.video, cfg.net.name, cfg.net.patch_t, cfg.net.patch, cfg.net.patch, cfg.N, cfg.T,
                                  cfg.net.C0, cfg.H, cfg.W, cfg.mask_frac * 100),
                   "conv_algo": "auto" if args.algo == 0 else "direct", "launch": "eager"},
        "roofline": roof,
        "worst_dense_conv_frac_of_mfma_peak": None if worst_conv is None else round(worst_conv, 4),
        "worst_pool_frac_of_hbm_peak": None if worst_pool is None else round(worst_pool, 4),
        "layers": sorted(rows, key=lambda r: (r["layer"], r["call"])),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = video_cpu_baseline(cfg, wl, args.forward_only)
    print(json.dumps(out))


def measured_traffic(config, dtype, call, layer):
    """HBM bytes one launch of (call, layer) moved, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    summary committed under profiles/ for this workload (bench.py cannot collect counters itself);
    None when no summary covers the workload or the call."""
    name = "bench_config%d_%s_hbm_traffic.md" % (config, {"f32": "fp32"}.get(dtype, dtype))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", name)
    if not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 5 and cells[0] == call and cells[1] == str(layer):
            return {"fetched_bytes": int(float(cells[2]) * (1 << 20)), "written_bytes": int(float(cells[3]) * (1 << 20)),
                    "bytes": int(float(cells[4]) * (1 << 20)), "source": "profiles/" + name}
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--dtype", default=None)
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--image-size", type=int, default=0,
                    help="override the labelled image to S x S pixels (the paper's image-size sweep)")
    ap.add_argument("--mask-frac", type=float, default=-1.0,
                    help="override the fraction of labelled pixels whose errors are kept (Sec. 4.3: the cost "
                         "of the backward pass does not depend on it)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of the step captured in a HIP graph (per-call rates then come from an "
                         "eager pass before the timed region)")
    ap.add_argument("--algo", type=int, default=0)
    ap.add_argument("--no-fuse", action="store_true",
                    help="backward: pool gradient and non-linearity backward + bias gradient as separate calls")
    ap.add_argument("--compare-fast-scanning", action="store_true",
                    help="also time the forward pass of the comparison method (fast scanning: strided layers run once "
                         "per starting offset on fragments) on the same workload; reported under \"fast_scanning\"")
    ap.add_argument("--video", type=int, default=-1,
                    help="measure video workload I (3-D convolution and pooling) instead of an image configuration")
    ap.add_argument("--layers", action="store_true", help="print the per-call table to stderr")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a known-size reference "
                         "for scaling HBM byte counters collected with rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    if args.video >= 0:
        return main_video(args)

    import numpy as np
    import torch
    import paper_1412_4526_amd as dsk
    from workloads import CONFIGS, make_workload

    cfg = CONFIGS[args.config]
    if args.image_size > 0 or args.mask_frac >= 0:
        import dataclasses
        if args.image_size > 0:
            cfg = dataclasses.replace(cfg, H=args.image_size, W=args.image_size)
        if args.mask_frac >= 0:
            cfg = dataclasses.replace(cfg, mask_frac=args.mask_frac)
    dtype = args.dtype or cfg.dtype
    elem = 4 if dtype == "f32" else 2
    wl = make_workload(cfg.net, cfg.N, cfg.H, cfg.W, cfg.mask_frac, cfg.seed, positive_frac=cfg.positive_frac)
    dev = "cuda:0"
    dsk.dsk_set_conv_algo(args.algo)
    net = dsk.WholeImageNet(cfg.net, cfg.N, cfg.H, cfg.W, dtype, dev, train=not args.forward_only, fuse=not args.no_fuse)
    net.load_params(wl.weights, wl.biases)
    image = torch.from_numpy(wl.image).to(dev)
    labels = torch.from_numpy(wl.labels).to(dev)
    mask = torch.from_numpy(wl.mask).to(dev)

    def step():
        net.forward(image)
        if not args.forward_only:
            net.loss_backward(labels, mask)

    if args.calib_copy_mib > 0:
        src = torch.zeros(args.calib_copy_mib * (1 << 20) // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                  # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        # per-call events cannot be recorded into a graph: collect them from eager steps first
        net.timeline = []
        for _ in range(max(3, args.warmup)):
            step()
        torch.cuda.synchronize()
        timeline, net.timeline = net.timeline, None
        if args.forward_only:
            net.capture(image)
        else:
            net.capture(image, labels, mask)
        net.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            net.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    else:
        warm_event_pool(torch, 8192 + 2 * (3 * len(net.plan) + 4) * args.steps)
        net.timeline = []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        timeline, net.timeline = net.timeline, None

    pixels = cfg.N * cfg.H * cfg.W
    # per-call device time from the events recorded inside the timed region
    per = {}
    for tag, layer, e0, e1 in timeline:
        per.setdefault((tag, layer), []).append(e0.elapsed_time(e1))
    costs = layer_costs(net, elem)
    rows = []
    for key, ms in per.items():
        avg = sum(ms) / len(ms)
        c = costs[key]
        p = net.plan[key[1]] if 0 <= key[1] < len(net.plan) else None
        row = {"call": key[0], "layer": key[1], "ms": round(avg, 4)}
        if p is not None:
            row["shape"] = "C%d K%d k%d d%d %dx%d" % (p.C, p.K, p.k, p.d, p.H, p.W)
        if c["flops"] > 0:
            row["tflops"] = round(c["flops"] / avg / 1e9, 2)
            row["intensity"] = round(c["flops"] / c["bytes"], 1)
        row["gbs"] = round(c["bytes"] / avg / 1e6, 1)
        rows.append(row)
    if args.layers:
        for r in sorted(rows, key=lambda r: -r["ms"]):
            sys.stderr.write(json.dumps(r) + "\n")

    # roofline of the dominant call
    dom = max(rows, key=lambda r: r["ms"])
    c = costs[(dom["call"], dom["layer"])]
    peak_mfma = PEAK_FP32_MFMA if dtype == "f32" else PEAK_BF16_MFMA
    ridge = peak_mfma * 1e3 / PEAK_HBM          # flop per byte where the two roofs meet
    if c["flops"] > 0 and c["flops"] / c["bytes"] >= ridge:
        roof = {"bound": "mfma", "achieved": dom["tflops"], "peak": peak_mfma, "unit": "TFLOP/s",
                "frac": round(dom["tflops"] / peak_mfma, 4)}
    else:
        roof = {"bound": "hbm", "achieved": dom["gbs"], "peak": PEAK_HBM, "unit": "GB/s",
                "frac": round(dom["gbs"] / PEAK_HBM, 4)}
    tr = measured_traffic(args.config, dtype, dom["call"], dom["layer"])
    roof["traffic"] = None if tr is None else tr["bytes"]        # HBM bytes per launch (fetched + written)
    roof["traffic_detail"] = tr
    roof["algorithmic_bytes"] = int(c["bytes"])
    roof["algorithmic_flops"] = int(c["flops"])
    roof["kernel"] = "%s layer %d (%s)" % (dom["call"], dom["layer"], dom.get("shape", ""))
    roof["ms"] = dom["ms"]

    # dense contractions only (every 3x3 / 4x4 / 5x5 layer with >= 32 input channels has an arithmetic
    # intensity in the hundreds); the first layer (3 input channels) and the 1x1 layers sit near or
    # below the ridge and are listed with both rates in "layers"
    worst_conv = min((r["tflops"] / peak_mfma for r in rows
                      if "tflops" in r and r["intensity"] >= kDenseIntensity), default=None)
    worst_pool = min((r["gbs"] / PEAK_HBM for r in rows if "pool" in r["call"]), default=None)

    vs_baseline = None
    if args.config == 5 and dtype == "f32" and args.image_size == 0:
        paper_ms = PAPER_PLAIN_CNN1_MS["fwd" if args.forward_only else "fwd+bwd"]
        vs_baseline = round((pixels * args.steps / dt) / (pixels / (paper_ms * 1e-3)), 2)
    out = {
        "metric": "labelled pixels/s whole-image %s" % ("fwd" if args.forward_only else "fwd+bwd"),
        "value": pixels * args.steps / dt, "unit": "labelled pixels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": vs_baseline, "dtype": dtype,
        "data": "synthetic",
        "config": {"workload": "configs[%d]: %s patch %d, %dx%dx%dx%d image, mask %.0f%%"
                               % (args.config, cfg.net.name, cfg.net.patch, cfg.N, cfg.net.C0, cfg.H, cfg.W,
                                  cfg.mask_frac * 100),
                   "conv_algo": "auto" if args.algo == 0 else "direct",
                   "launch": "hip graph replay" if args.graph else "eager"},
        "roofline": roof,
        "worst_dense_conv_frac_of_mfma_peak": None if worst_conv is None else round(worst_conv, 4),
        "worst_pool_frac_of_hbm_peak": None if worst_pool is None else round(worst_pool, 4),
        # conv calls left out of the dense minimum (first layer, 1x1 layers): both fractions, the larger one binds
        "conv_calls_near_or_below_the_ridge": [
            {"call": r["call"], "layer": r["layer"], "shape": r.get("shape", ""), "intensity": r["intensity"],
             "frac_of_mfma_peak": round(r["tflops"] / peak_mfma, 4), "frac_of_hbm_peak": round(r["gbs"] / PEAK_HBM, 4)}
            for r in sorted(rows, key=lambda r: (r["layer"], r["call"])) if "tflops" in r and r["intensity"] < kDenseIntensity],
        "layers": sorted(rows, key=lambda r: (r["layer"], r["call"])),
    }
    if args.compare_fast_scanning:
        fs = dsk.FastScanNet(cfg.net, cfg.N, cfg.H, cfg.W, dtype, dev)
        fs.load_params(wl.weights, wl.biases)
        for _ in range(args.warmup):
            fs.forward(image)
        torch.cuda.synchronize()
        fs.timeline = []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fs.forward(image)
        torch.cuda.synchronize()
        fdt = time.perf_counter() - t0
        fper = {}
        for tag, layer, e0, e1 in fs.timeline:
            fper.setdefault((tag, layer), []).append(e0.elapsed_time(e1))
        out["fast_scanning"] = {
            "what": "forward pass of the comparison method on the same workload (it has no backward pass)",
            "ms_per_step": fdt / args.steps * 1e3, "labelled_pixels_per_s": pixels * args.steps / fdt,
            "fragments_per_image_after_each_layer": fs.fragments(),
            "layers": [{"call": k[0], "layer": k[1], "ms": round(sum(v) / len(v), 4)} for k, v in sorted(fper.items(), key=lambda kv: kv[0][1])]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl, args.forward_only)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
