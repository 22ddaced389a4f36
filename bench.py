#!/usr/bin/env python3
"""Benchmark of the SqueezeNet v1.0 forward path on one MI355X.

One "step" is one pass of the whole hot path -- sq_squeezenet_forward: conv1, three max
poolings, eight fire layers, conv10, global average pooling, softmax -- over one batch of
synthetic images already resident in HBM (the call is sq_squeezenet_forward_packed: the kernels
were re-ordered once by sq_pack_weights before any timing, as the paper re-orders its kernels offline).  The workload is the full network at batch 64
(fp32, uniform[0,1) inputs, He-normal kernels, seed 3); batch 1 (seed 2) is timed beside it.

Prints ONE JSON line.  `value` is images/s at batch 64 over the timed region: exactly
--steps calls of sq_squeezenet_forward_packed between two device synchronisations, nothing else
on the stream.  Right after it the same number of steps is run again with the library's
per-launch HIP events switched on (sq_profile_begin/end: an event pair around every kernel,
recorded on the stream the kernels run on); that pass gives the per-kernel and per-layer
durations behind `roofline` and `layers`, and its own step time is reported as
`ms_per_step_with_events` (the events keep consecutive kernels from overlapping their
launch, so it is a little slower).  `cpu_baseline` is the CPU oracle timed on the host
cores on a bounded sample of the same workload.

`reduced_precision` times the same network through sq_squeezenet_forward_bf16 (bfloat16
feature maps and kernels, fp32 sums: the counterpart of the paper's relaxed-precision mode)
on the same images, and reports how often it predicts the class the fp32 network predicts.

`energy` is the analogue of the paper's power table (section "Power Consumption"): the GPU's
own power sensor is sampled while idle (before any kernel runs) and while forward passes run
back to back for --energy-seconds; energy per image = power x time per image, given both for
the total power and for the differential (load minus idle) power, as the paper does.

`python bench.py --calibrate-copy` instead runs a plain 1 GiB device-to-device copy a few
times and exits; it is the known-size kernel that the HBM byte counters are scaled by.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP32_MFMA_PEAK_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0
FLOP_PER_IMAGE = 2 * 832_667_936  # 2 x multiply-accumulates of the 26 convolutions


def kernel_sources_hash():
    """SHA-256 over the kernel sources (csrc/*.hip, *.h, *.inc), in name order: identifies what the library was built from."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_1611_07151_amd", "csrc", "*"))):
        if path.endswith((".hip", ".h", ".inc")):
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    return h.hexdigest()


def power_sensor():
    """Path of the GPU's power reading (hwmon, microwatts), or None."""
    import glob
    for pat in ("power1_input", "power1_average"):
        hits = sorted(glob.glob(f"/sys/class/drm/card*/device/hwmon/hwmon*/{pat}"))
        if hits:
            return hits[0]
    return None


def sample_power(path, seconds, work, settle=0.0):
    """Calls work() over and over for `seconds` and reads the sensor between calls (at most every
    5 ms); readings of the first `settle` seconds are dropped.  Mean in watts."""
    vals, t0, last = [], time.perf_counter(), 0.0
    while True:
        now = time.perf_counter() - t0
        if now >= seconds + settle:
            break
        work()
        if now - last >= 0.005:
            last = now
            try:
                v = int(open(path).read())
            except (OSError, ValueError):
                continue
            if now >= settle:
                vals.append(v * 1e-6)
    if not vals:
        return dict(mean_w=float("nan"), samples=0)
    return dict(mean_w=sum(vals) / len(vals), samples=len(vals))


def layer_sweep(sq, synth, torch, mode, B, net="squeezenet", only=None):
    """Times every convolution shape of a network on its own at batch B; mode "f32" / "bf16" (NCHW inputs of that
    type, fp32 accumulate and output) or "blocked" (the reduced-precision kernels on blocked bfloat16 maps)."""
    dt_in = torch.bfloat16 if mode == "bf16" else torch.float32
    esz = 2 if mode == "bf16" else 4
    out_note = "bfloat16 maps and kernels, fp32 accumulate" if mode == "blocked" else f"{mode} inputs, fp32 accumulate/output"
    gen = torch.Generator(device="cuda").manual_seed(4)
    layers, total_flop, total_us, total_bytes = {}, 0.0, 0.0, 0.0
    net_layers = synth.conv_layers() if net == "squeezenet" else synth.second_network_layers()
    if only:
        net_layers = [l for l in net_layers if only in l[0]]
    for name, cin, cout, k, s_, p_, h in net_layers:
        ho = (h + 2 * p_ - k) // s_ + 1
        if mode == "blocked":
            # the same shape through the reduced-precision kernels: blocked bfloat16 in and out, kernels packed ahead
            xf = torch.randn((B, cin, h, h), device="cuda", generator=gen)
            wf = torch.randn((cout, cin, k, k), device="cuda", generator=gen) * (2.0 / (cin * k * k)) ** 0.5
            b = torch.rand(cout, device="cuda", generator=gen) * 0.2 - 0.1
            if k == 7:
                wp = sq.sq_blocked_pack_kernels7(wf)
                run = lambda: sq.sq_blocked_conv7s2_forward(xf, wp, b, cout, p_, True, out=outm)
                in_bytes = 4.0 * B * cin * h * h
            elif sq.lib.sq_blocked_kernel_bytes(cout, cin, k) and cin % 16 == 0 and k in (1, 3, 5) and s_ == 1 and p_ == k // 2:
                xm = sq.sq_blocked_pack(xf)
                wp = sq.sq_blocked_pack_kernels(wf)
                run = lambda: sq.sq_blocked_conv2d_forward(xm, wp, b, cin, cout, k, p_, True, out=outm)
                in_bytes = 2.0 * B * cin * h * h
            else:
                continue                      # a shape the blocked kernels do not cover
            outm = torch.empty((B, (cout + 7) // 8, ho, ho, 8), device="cuda", dtype=torch.bfloat16)
            for _ in range(3):
                run()
            sq.sq_profile_begin(64)
            for _ in range(10):
                run()
            recs = sq.sq_profile_end()
            us = sum(r["ms"] for r in recs) / 10 * 1e3
            flop = 2.0 * B * cout * ho * ho * cin * k * k
            byts = in_bytes + 2.0 * cout * cin * k * k + 2.0 * B * cout * ho * ho
            layers[name] = dict(us=round(us, 1), tflops=round(flop / us / 1e6, 1), gbs=round(byts / us / 1e3),
                                kernel=recs[0]["name"].split("|")[1])
            total_flop += flop
            total_us += us
            total_bytes += byts
            del xf, wf, outm
            continue
        x = torch.randn((B, cin, h, h), device="cuda", generator=gen).to(dt_in)
        w = (torch.randn((cout, cin, k, k), device="cuda", generator=gen) * (2.0 / (cin * k * k)) ** 0.5).to(dt_in)
        b = torch.rand(cout, device="cuda", generator=gen) * 0.2 - 0.1
        out = torch.empty((B, cout, ho, ho), device="cuda")
        scratch = torch.empty(max(256, sq.sq_conv2d_workspace_bytes(cin, cout, k, s_, p_),
                                  sq.sq_conv2d_strided_workspace_bytes(B, cin, h, h, cout, k, s_, p_),
                                  sq.sq_conv2d_bf16_workspace_bytes(B, cin, h, h, cout, k, s_, p_) if mode == "bf16" else 0),
                              device="cuda", dtype=torch.uint8)
        for _ in range(3):
            sq.sq_conv2d_forward_ws(x, w, b, s_, p_, True, out=out, workspace=scratch)
        sq.sq_profile_begin(64)
        for _ in range(10):
            sq.sq_conv2d_forward_ws(x, w, b, s_, p_, True, out=out, workspace=scratch)
        recs = sq.sq_profile_end()
        us = sum(r["ms"] for r in recs) / 10 * 1e3   # kernel transform included where one runs
        flop = 2.0 * B * cout * ho * ho * cin * k * k
        byts = esz * (B * cin * h * h + cout * cin * k * k) + 4.0 * B * cout * ho * ho
        layers[name] = dict(us=round(us, 1), tflops=round(flop / us / 1e6, 1), gbs=round(byts / us / 1e3),
                            kernel=max(recs, key=lambda r: r["ms"])["name"].split("|")[1])
        total_flop += flop
        total_us += us
        total_bytes += byts
        del x, w, out
    return {"metric": f"per-layer convolution sweep, batch {B}, {out_note}",
            "value": round(total_flop / total_us / 1e6, 2), "unit": "TFLOP/s (all layers)",
            "gbs_all_layers": round(total_bytes / total_us / 1e3),
            "n_gpus": 1, "dtype": "bf16" if mode == "blocked" else mode, "data": "synthetic",
            "config": {"workload": f"{len(net_layers)} convolution shapes ({net}) at batch {B}"},
            "total_us": round(total_us, 1), "layers": layers}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--print-kernel-hash", action="store_true", help="print the hash of the kernel sources and exit")
    ap.add_argument("--layer-sweep", choices=["f32", "bf16", "blocked"], default=None,
                    help="instead of the network: time every convolution shape on its own at --batch "
                         "(workload 5 is --layer-sweep bf16 --batch 256) and print one JSON line; "
                         "'blocked' = the reduced-precision kernels on blocked bfloat16 maps")
    ap.add_argument("--only", default=None, help="with --layer-sweep: only the layers whose name contains this")
    ap.add_argument("--net", choices=["squeezenet", "second"], default="squeezenet",
                    help="layer list of --layer-sweep: SqueezeNet's 26 convolutions, or the five of a second CNN "
                         "(11x11 stride 4, 5x5, 3x3)")
    ap.add_argument("--energy-seconds", type=float, default=3.0,
                    help="length of each power-sampling window (0 = leave the energy measurement out)")
    ap.add_argument("--skip-reduced", action="store_true", help="leave the reduced-precision (bf16) network out")
    ap.add_argument("--skip-batch1", action="store_true", help="leave the batch-1 timing out (for profiler runs)")
    ap.add_argument("--skip-sweep", action="store_true",
                    help="leave the per-layer sweep at batch 256 with bfloat16 inputs (workload 5) out")
    ap.add_argument("--cpu-sample", type=int, default=64,
                    help="images of the workload the CPU oracle is timed on (0 = skip)")
    args = ap.parse_args()
    if args.print_kernel_hash:
        print(kernel_sources_hash())
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (images are independent, so more GPUs "
              "would each take a slice of the batch with no communication); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_1611_07151_amd as sq
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    K, W, B = args.steps, args.warmup, args.batch

    if args.calibrate_copy:
        n = 1 << 28                                   # 2^28 floats = 1 GiB read + 1 GiB written
        src = torch.ones(n, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch elementwise copy", "bytes_read": 4 * n, "bytes_written": 4 * n,
                          "launches": 5}))
        return 0

    sensor = power_sensor()
    idle_w = None
    if sensor and args.energy_seconds > 0 and not args.layer_sweep:
        torch.cuda.synchronize()                       # context is up, nothing has run yet
        idle_w = sample_power(sensor, min(2.0, args.energy_seconds), lambda: time.sleep(0.01))

    if args.layer_sweep:
        print(json.dumps(layer_sweep(sq, synth, torch, args.layer_sweep, B, args.net, args.only)))
        return 0

    def setup(seed, n):
        cfg = synth.config_squeezenet(seed=seed, n=n)
        x = torch.from_numpy(cfg["x"]).cuda()
        params = [torch.from_numpy(p).cuda() for p in cfg["params"]]
        ws = torch.empty(sq.sq_squeezenet_workspace_bytes(n), device="cuda", dtype=torch.uint8)
        probs = torch.empty((n, 1000), device="cuda")
        # kernels re-ordered once, ahead of time and outside every timed region (the paper re-orders its kernels
        # offline too, section "Zero-overhead Vectorization"); the forward pass only reads them
        packed = sq.sq_pack_weights(params, sq.SQ_F32)
        return cfg, x, (params, packed), ws, probs

    def timed(x, params, ws, probs, steps, profile):
        if profile:
            sq.sq_profile_begin(steps * 48)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            sq.sq_squeezenet_forward_packed(x, params[0], params[1], workspace=ws, probs=probs)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dt, (sq.sq_profile_end() if profile else None)

    # ---------------------------------------------------------------- batch 64 (the metric)
    cfg, x, params, ws, probs = setup(3, B)
    sq.sq_init()
    for _ in range(W):
        sq.sq_squeezenet_forward_packed(x, params[0], params[1], workspace=ws, probs=probs)
    dt, _ = timed(x, params, ws, probs, K, False)                # THE timed region
    dt_events, recs = timed(x, params, ws, probs, K, True)       # same steps again, with per-launch events
    params, packed32 = params
    ms_per_step = dt / K * 1e3
    images_per_s = B * K / dt
    assert torch.isfinite(probs).all()

    kernels, stages = {}, {}
    for r in recs:
        stage, kernel = r["name"].split("|")
        for table, key in ((kernels, kernel), (stages, stage)):
            e = table.setdefault(key, dict(launches=0, ms=0.0, flops=0.0, bytes=0.0, mfma_flops=0.0))
            for f in ("launches", "ms", "flops", "bytes", "mfma_flops"):
                e[f] += r[f]
    dom_name, dom = max(kernels.items(), key=lambda kv: kv[1]["ms"])
    dom_ms = dom["ms"] / dom["launches"]
    achieved = dom["flops"] / dom["launches"] / (dom_ms * 1e-3) / 1e12
    # HBM bytes per launch of the dominant kernel from the rocprofv3 counter runs summarised under profiles/: only
    # valid for the kernels they were measured on, so the file carries a hash of the kernel sources and a figure
    # measured on other sources is not reported
    traffic, traffic_note = None, "profiles/traffic.json has no entry for this kernel"
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("kernel_sources_sha256") != kernel_sources_hash():
            traffic_note = "profiles/traffic.json was measured on other kernel sources than the ones built here"
        elif dom_name in tj.get("bytes_per_launch", {}):
            traffic, traffic_note = tj["bytes_per_launch"][dom_name], "FETCH_SIZE + WRITE_SIZE per launch, scaled by the copy calibration (profiles/hbm_traffic.md)"
    executed = dom["mfma_flops"] / dom["launches"] / (dom_ms * 1e-3) / 1e12
    roofline = dict(bound="mfma", achieved=round(achieved, 2), peak=FP32_MFMA_PEAK_TFLOPS,
                    unit="TFLOP/s", frac=round(achieved / FP32_MFMA_PEAK_TFLOPS, 4), traffic=traffic,
                    traffic_note=traffic_note,
                    executed_tflops=round(executed, 2), executed_frac=round(executed / FP32_MFMA_PEAK_TFLOPS, 4),
                    note="achieved/frac count the layer definition's 2 x MACs (algorithmic); executed_* count the "
                         "operations the kernel's MFMA instructions really issue (padding included; the "
                         "minimal-filtering part forms 16 products where the definition has 36) = matrix-core utilisation",
                    kernel=dom_name, launches_per_step=dom["launches"] / K,
                    avg_launch_us=round(dom_ms * 1e3, 2),
                    flop_per_launch=dom["flops"] / dom["launches"],
                    mfma_flop_per_launch=dom["mfma_flops"] / dom["launches"],
                    share_of_gpu_time=round(dom["ms"] / sum(k["ms"] for k in kernels.values()), 3))
    all_mfma = sum(k["mfma_flops"] for k in kernels.values()) / K
    all_ms = sum(k["ms"] for k in kernels.values()) / K
    layers = {}
    for name, e in stages.items():
        us = e["ms"] / K * 1e3
        layers[name] = dict(us=round(us, 1),
                            tflops=round(e["flops"] / K / us / 1e6, 1) if e["flops"] else None,
                            executed_tflops=round(e["mfma_flops"] / K / us / 1e6, 1) if e["flops"] else None,
                            gbs=round(e["bytes"] / K / us / 1e3, 0))
    # One row per module of the network (a fire layer = its squeeze and both expands; the classifier = conv10, average
    # pooling and softmax): algorithmic TFLOP/s against the fp32 matrix peak and algorithmic GB/s against the HBM peak.
    modules = {}
    for name, e in stages.items():
        mod = name.split("/")[0] if name.startswith("fire") else "classifier" if name in ("conv10", "avgpool", "softmax", "avgpool+softmax") else name
        m = modules.setdefault(mod, dict(us=0.0, flops=0.0, bytes=0.0))
        m["us"] += e["ms"] / K * 1e3
        m["flops"] += e["flops"] / K
        m["bytes"] += e["bytes"] / K
    for m in modules.values():
        tf, gb = m["flops"] / m["us"] / 1e6, m["bytes"] / m["us"] / 1e3
        m.update(us=round(m["us"], 1), tflops=round(tf, 1), pct_fp32_mfma_peak=round(100 * tf / FP32_MFMA_PEAK_TFLOPS, 1),
                 gbs=round(gb), pct_hbm_peak=round(100 * gb / HBM_PEAK_GBS, 1))
        del m["flops"], m["bytes"]
    # Every launch that does convolution work counts; the squeeze layers behind a max pooling do that pooling
    # while they read their input (kernel names "pool3s2+...", or "poolrows+..." where the layer before has already
    # pooled the columns), so the pooling time is in this figure too.
    conv_ms = sum(e["ms"] for e in stages.values() if e["flops"]) / K
    conv_tflops = B * FLOP_PER_IMAGE / (conv_ms * 1e-3) / 1e12
    pooling = [r for r in recs if r["name"].split("|")[1].startswith(("pool3s2+", "poolrows+"))]
    plain_ms = conv_ms - sum(r["ms"] for r in pooling) / K
    plain_tflops = (B * FLOP_PER_IMAGE - sum(r["flops"] for r in pooling) / K) / (plain_ms * 1e-3) / 1e12

    # ---------------------------------------------------------------- batch 1
    k1, dt1, dt1g, graph_ok, launches1 = 1, float("nan"), float("nan"), None, None
    if not args.skip_batch1:
        cfg1, x1, params1, ws1, probs1 = setup(2, 1)
        for _ in range(20):
            sq.sq_squeezenet_forward_packed(x1, params1[0], params1[1], workspace=ws1, probs=probs1)
        k1 = max(200, K)
        dt1, _ = timed(x1, params1, ws1, probs1, k1, False)
        _, recs1 = timed(x1, params1, ws1, probs1, 10, True)
        launches1 = sum(r["launches"] for r in recs1) // 10
        params1, packed1_32 = params1
        # the same batch-1 pass replayed from a HIP graph (the library call allocates nothing and
        # does not synchronise, so the caller can capture it); checked against the eager result
        eager = probs1.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            sq.sq_squeezenet_forward_packed(x1, params1, packed1_32, workspace=ws1, probs=probs1)
            with torch.cuda.graph(graph, stream=side):
                sq.sq_squeezenet_forward_packed(x1, params1, packed1_32, workspace=ws1, probs=probs1)
        torch.cuda.current_stream().wait_stream(side)
        probs1.zero_()
        graph.replay()
        torch.cuda.synchronize()
        graph_ok = bool(torch.equal(probs1, eager))
        t0 = time.perf_counter()
        for _ in range(k1):
            graph.replay()
        torch.cuda.synchronize()
        dt1g = time.perf_counter() - t0

    # ---------------------------------------------------------------- reduced precision (bf16 maps and kernels)
    # the same network through sq_squeezenet_forward_bf16: kernels re-ordered once ahead of time, fp32 image in
    reduced = None
    if not args.skip_reduced:
        packed = sq.sq_squeezenet_bf16_pack_params(params)
        ws16 = torch.empty(sq.sq_squeezenet_bf16_workspace_bytes(B), device="cuda", dtype=torch.uint8)
        probs16 = torch.empty((B, 1000), device="cuda")

        def timed16(xx, pp, pk, ww, oo, steps, profile):
            if profile:
                sq.sq_profile_begin(steps * 48)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                sq.sq_squeezenet_forward_bf16(xx, pp, pk, workspace=ww, probs=oo)
            torch.cuda.synchronize()
            dt_ = time.perf_counter() - t0
            return dt_, (sq.sq_profile_end() if profile else None)

        for _ in range(W):
            sq.sq_squeezenet_forward_bf16(x, params, packed, workspace=ws16, probs=probs16)
        dt16, _ = timed16(x, params, packed, ws16, probs16, K, False)
        _, recs16 = timed16(x, params, packed, ws16, probs16, K, True)
        layers16 = {}
        for r in recs16:
            st = r["name"].split("|")[0]
            e = layers16.setdefault(st, dict(us=0.0, flops=0.0, bytes=0.0, kernel=r["name"].split("|")[1]))
            e["us"] += r["ms"] / K * 1e3
            e["flops"] += r["flops"] / K
            e["bytes"] += r["bytes"] / K
        for e in layers16.values():
            e["tflops"] = round(e.pop("flops") / e["us"] / 1e6, 1)
            e["gbs"] = round(e.pop("bytes") / e["us"] / 1e3)
            e["us"] = round(e["us"], 1)
        # agreement with the fp32 network on the images of this batch (class means decide the prediction)
        _, t32 = sq.sq_squeezenet_forward(x, params, workspace=ws, want_taps=True)
        _, t16 = sq.sq_squeezenet_forward_bf16(x, params, packed, workspace=ws16, want_taps=True)
        m32, m16 = t32["means"].double(), t16["means"].double()
        rel = ((m16 - m32).abs() / m32.std(dim=1, keepdim=True))
        reduced = dict(images_per_s=round(B * K / dt16, 1), ms_per_step=round(dt16 / K * 1e3, 4),
                       speedup_vs_fp32=round(dt / dt16, 3), dtype="bf16 maps and kernels, fp32 accumulate",
                       top1_agreement_with_fp32=round(float((m16.argmax(1) == m32.argmax(1)).double().mean()), 4),
                       class_mean_error_over_spread=dict(max=round(float(rel.max()), 4),
                                                         rms=round(float((rel ** 2).mean().sqrt()), 5)),
                       conv_tflops=round(B * FLOP_PER_IMAGE / (sum(e["us"] for e in layers16.values() if e["tflops"]) * 1e-6) / 1e12, 1),
                       layers=layers16)
        del t32, t16
        if not args.skip_batch1:
            packed1 = sq.sq_squeezenet_bf16_pack_params(params1)
            ws161 = torch.empty(sq.sq_squeezenet_bf16_workspace_bytes(1), device="cuda", dtype=torch.uint8)
            for _ in range(20):
                sq.sq_squeezenet_forward_bf16(x1, params1, packed1, workspace=ws161, probs=probs1)
            d1, _ = timed16(x1, params1, packed1, ws161, probs1, k1, False)
            reduced["batch1_ms"] = round(d1 / k1 * 1e3, 4)
            reduced["batch1_images_per_s"] = round(k1 / d1, 1)

    # ---------------------------------------------------------------- energy per image
    energy = None
    if idle_w is not None:
        def run_for(xx, pp, ww, oo, n, packed_kernels=None):
            def burst():
                for _ in range(8):
                    if packed_kernels is None:
                        sq.sq_squeezenet_forward_packed(xx, pp[0], pp[1], workspace=ww, probs=oo)
                    else:
                        sq.sq_squeezenet_forward_bf16(xx, pp, packed_kernels, workspace=ww, probs=oo)
                torch.cuda.synchronize()
            load = sample_power(sensor, args.energy_seconds, burst, settle=0.5)
            t0, reps = time.perf_counter(), 0
            while time.perf_counter() - t0 < 0.5:
                burst()
                reps += 8
            s_per_image = (time.perf_counter() - t0) / (reps * n)
            return dict(load_w=round(load["mean_w"], 1), differential_w=round(load["mean_w"] - idle_w["mean_w"], 1),
                        samples=load["samples"], ms_per_image=round(s_per_image * 1e3, 5),
                        j_per_image_total=round(load["mean_w"] * s_per_image, 6),
                        j_per_image_differential=round((load["mean_w"] - idle_w["mean_w"]) * s_per_image, 6))
        energy = dict(source=sensor + " (GPU package power, microwatts)", idle_w=round(idle_w["mean_w"], 1),
                      idle_samples=idle_w["samples"], window_s=args.energy_seconds)
        energy[f"batch{B}"] = run_for(x, (params, packed32), ws, probs, B)
        if not args.skip_batch1:
            energy["batch1"] = run_for(x1, (params1, packed1_32), ws1, probs1, 1)
        if reduced is not None:
            energy[f"batch{B}_reduced_precision"] = run_for(x, params, ws16, probs16, B, packed)

    # ---------------------------------------------------------------- CPU oracle baseline
    cpu = None
    if args.cpu_sample > 0:
        import oracle
        n = min(args.cpu_sample, B)
        # the same call again until ten seconds have passed (at most eight times): a bounded sample, long enough to time
        calls, cdt = 0, 0.0
        while calls < 8 and cdt < 10.0:
            t0 = time.perf_counter()
            ref = oracle.squeezenet(cfg["x"][:n], cfg["params"])
            cdt += time.perf_counter() - t0
            calls += 1
        got = probs[:n].cpu().numpy()
        err = float(np.max(np.abs(got - ref) / (1 + np.abs(ref))))
        cpu = dict(value=round(n * calls / cdt, 3), unit="images/s", cores=oracle.num_threads(), kind="oracle",
                   sample=f"first {n} images of the batch-{B} workload, {calls} oracle.squeezenet calls "
                          f"({cdt:.1f} s)", gflops=round(n * calls * FLOP_PER_IMAGE / cdt / 1e9, 2),
                   max_scaled_error_gpu_vs_oracle=err)
        # the paper's own baseline is one image on one core ("sequential"): the batch-1 workload on a single thread
        threads = oracle.num_threads()
        cfg_one = synth.config_squeezenet(seed=2, n=1)
        oracle.set_num_threads(1)
        try:
            t0 = time.perf_counter()
            oracle.squeezenet(cfg_one["x"], cfg_one["params"])
            sdt = time.perf_counter() - t0
        finally:
            oracle.set_num_threads(threads)
        cpu["single_thread"] = dict(seconds_per_image=round(sdt, 3), images_per_s=round(1.0 / sdt, 3), cores=1,
                                    gflops=round(FLOP_PER_IMAGE / sdt / 1e9, 3),
                                    sample="the batch-1 workload (seed 2), one image, one thread")

    # ---------------------------------------------------------------- workload 5: per-layer sweep, batch 256, bf16 inputs
    sweep = None
    if not args.skip_sweep:
        del x, ws
        torch.cuda.empty_cache()
        sw = layer_sweep(sq, synth, torch, "bf16", 256)
        sweep = dict(workload="every convolution shape of the network on its own at batch 256, bfloat16 inputs and kernels "
                              "(NCHW), fp32 accumulate and output, seed 4",
                     tflops_all_layers=sw["value"], gbs_all_layers=sw["gbs_all_layers"], total_us=sw["total_us"],
                     pct_hbm_peak=round(100 * sw["gbs_all_layers"] / HBM_PEAK_GBS, 1),
                     slowest={k: v for k, v in sorted(sw["layers"].items(), key=lambda kv: -kv[1]["us"])[:3]})
        # the same shapes on the bf16 matrix instructions: blocked bfloat16 maps in and out, kernels packed ahead
        # (the layout and kernels of the reduced-precision network), each layer on its own
        sb = layer_sweep(sq, synth, torch, "blocked", 256)
        sweep["on_bf16_mfma_blocked_layout"] = dict(
            tflops_all_layers=sb["value"], gbs_all_layers=sb["gbs_all_layers"], total_us=sb["total_us"],
            pct_bf16_mfma_peak=round(100 * sb["value"] / 2500.0, 1), pct_hbm_peak=round(100 * sb["gbs_all_layers"] / HBM_PEAK_GBS, 1),
            slowest={k: v for k, v in sorted(sb["layers"].items(), key=lambda kv: -kv[1]["us"])[:3]})

    out = {
        "metric": "SqueezeNet v1.0 forward images/sec at batch 64 (conv TFLOP/s and % fp32 MFMA peak beside it)",
        "value": round(images_per_s, 1), "unit": "images/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"full SqueezeNet v1.0 forward, batch {B}, fp32 NCHW, 3x224x224 "
                               "uniform[0,1) inputs, He-normal kernels, seed 3", "batch": B},
        "conv_tflops": round(conv_tflops, 2),
        "pct_fp32_mfma_peak": round(100 * conv_tflops / FP32_MFMA_PEAK_TFLOPS, 2),
        "conv_tflops_without_pooling_layers": dict(
            value=round(plain_tflops, 2), pct_fp32_mfma_peak=round(100 * plain_tflops / FP32_MFMA_PEAK_TFLOPS, 2),
            excluded=sorted({r["name"] for r in pooling}),
            note="the squeeze layers that max-pool their input on the way in are bound by reading that input, not by the MFMAs"),
        "end_to_end_tflops": round(B * FLOP_PER_IMAGE / (ms_per_step * 1e-3) / 1e12, 2),
        "batch1_images_per_sec": None if args.skip_batch1 else round(k1 / dt1, 1),
        "batch1_ms": None if args.skip_batch1 else round(dt1 / k1 * 1e3, 4),
        "batch1_launches": launches1,
        "batch1_graph_images_per_sec": None if args.skip_batch1 else round(k1 / dt1g, 1),
        "batch1_graph_matches_eager": graph_ok,
        "ms_per_step_with_events": round(dt_events / K * 1e3, 4),
        "mfma_utilisation_whole_pass": round(all_mfma / (all_ms * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS, 4),
        "roofline": roofline, "cpu_baseline": cpu, "energy": energy, "reduced_precision": reduced,
        "layer_sweep_bf16_batch256": sweep, "modules": modules, "layers": layers,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
