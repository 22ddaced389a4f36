#!/usr/bin/env python3
"""Times every tiling of the matrix-core convolution family on every SqueezeNet layer
shape and writes the per-shape winners as a C table (csrc/tuned_table.inc).

This is the counterpart of the paper's per-layer, per-device search for the best thread
granularity g (section "Optimizing Thread Granularity" and its table of optimal
granularities): here the searched quantity is the workgroup / wavefront tile shape.
Run on the GPU:  python paper_1611_07151_amd/tune.py [out.inc] [--batches 1,8,64,256]
then copy the file to paper_1611_07151_amd/csrc/tuned_table.inc and rebuild.

The three squeeze layers that follow a max-pooling layer are also timed with the pooling done
inside the convolution (sq_maxpool_conv2d_forward); those rows carry P = -1 and the pooled
extents.  --pooled-only keeps the other rows of an existing table and renews only these.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


# Shapes beside SqueezeNet's: the stride-1 form in which the second network's 11x11 stride-4 layer runs
# (48 space-to-depth layers of 57x57, 3x3 kernels, no padding), and that network's stride-1 layers.
EXTRA_LAYERS = [("c1/s2d", 48, 96, 3, 1, 0, 57), ("c2_5x5p2", 96, 256, 5, 1, 2, 27), ("c3_3x3p1", 256, 384, 3, 1, 1, 13),
                ("c4_3x3p1", 384, 384, 3, 1, 1, 13), ("c5_3x3p1", 384, 256, 3, 1, 1, 13)]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("out", nargs="?", default=os.path.join(ROOT, "paper_1611_07151_amd", "csrc", "tuned_table.inc"))
    ap.add_argument("--batches", default="1,8,64,256")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--pooled-only", action="store_true")
    args = ap.parse_args()

    import torch

    import paper_1611_07151_amd as sq
    import synth

    nv = sq.sq_conv_variant_count()
    names = [sq.sq_conv_variant_name(i) for i in range(nv)]
    rows, report = [], []

    def gpu_us(call):
        # GPU time of the launches themselves (the library's per-launch events)
        call()
        torch.cuda.synchronize()
        sq.sq_profile_begin(4 * args.reps + 4)
        for _ in range(args.reps):
            call()
        torch.cuda.synchronize()
        return sum(r["ms"] for r in sq.sq_profile_end()) / args.reps * 1e3

    for N in [int(b) for b in args.batches.split(",")]:
        # squeeze layers behind a pooling layer: (name, Cin, Cout, extent before pooling)
        for name, cin, cout, h in (("pool1+fire2/sq", 96, 16, 111), ("pool4+fire5/sq", 256, 32, 55), ("pool8+fire9/sq", 512, 64, 27)):
            hp = (h - 3) // 2 + 1
            x = torch.rand((N, cin, h, h), device="cuda")
            w = torch.randn((cout, cin, 1, 1), device="cuda") * (2.0 / cin) ** 0.5
            b = torch.rand(cout, device="cuda") * 0.2 - 0.1
            out = torch.empty((N, cout, hp, hp), device="cuda")
            timings = []
            for v in range(nv):
                try:
                    us = gpu_us(lambda: sq.sq_maxpool_conv2d_forward(x, w, b, True, out=out, algo=sq.SQ_ALGO_VARIANT0 + v))
                except sq.SqError:
                    continue
                timings.append((us, names[v]))
            timings.sort()
            pooled = sq.sq_maxpool(x)
            two_us = gpu_us(lambda: (sq.sq_maxpool(x), sq.sq_conv2d_forward_ex(pooled, w, b, 1, 0, True, out=out)))
            rows.append((1, 1, -1, cin, cout, hp, hp, N, timings[0][1], timings[0][1]))
            report.append(f"// N={N:3d} {name:14s} {cin:4d}->{cout:4d} k1 {hp:3d}x{hp:<3d}: best {timings[0][1]} {timings[0][0]:8.1f} us; "
                          f"worst {timings[-1][1]} {timings[-1][0]:8.1f} us; two launches {two_us:8.1f} us")
            print(report[-1], flush=True)
            del x, w, b, out, pooled
        if args.pooled_only:
            continue
        seen = set()
        for name, cin, cout, k, s, p, h in synth.conv_layers() + EXTRA_LAYERS:
            key = (k, s, p, cin, cout, h)
            if key in seen:
                continue
            seen.add(key)
            x = torch.rand((N, cin, h, h), device="cuda")
            w = torch.randn((cout, cin, k, k), device="cuda") * (2.0 / (cin * k * k)) ** 0.5
            b = torch.rand(cout, device="cuda") * 0.2 - 0.1
            ho = (h + 2 * p - k) // s + 1
            out = torch.empty((N, cout, ho, ho), device="cuda")
            ws = torch.empty(max(256, sq.sq_conv2d_workspace_bytes(cin, cout, k, s, p)), device="cuda", dtype=torch.uint8)
            flop = 2.0 * N * cout * ho * ho * cin * k * k
            timings = []
            for v in range(nv):
                try:
                    sq.sq_conv2d_forward_ws(x, w, b, s, p, True, out=out, algo=sq.SQ_ALGO_VARIANT0 + v, workspace=ws)
                except sq.SqError:
                    continue
                torch.cuda.synchronize()
                # GPU time of the launches themselves (the library's per-launch events): at small
                # batch the host cannot issue calls as fast as the kernels finish, so wall-clock
                # time per call would measure the host
                sq.sq_profile_begin(2 * args.reps + 4)
                for _ in range(args.reps):
                    sq.sq_conv2d_forward_ws(x, w, b, s, p, True, out=out, algo=sq.SQ_ALGO_VARIANT0 + v, workspace=ws)
                torch.cuda.synchronize()
                us = sum(r["ms"] for r in sq.sq_profile_end()) / args.reps * 1e3
                # does this tiling also run without scratch?
                try:
                    sq.sq_conv2d_forward_ex(x, w, b, s, p, True, out=out, algo=sq.SQ_ALGO_VARIANT0 + v)
                    plain = True
                except sq.SqError:
                    plain = False
                timings.append((us, names[v], plain))
            if not timings:
                continue
            timings.sort()
            best_us, best, _ = timings[0]
            worst_us, worst, _ = timings[-1]
            best_plain = [t for t in timings if t[2]][0][1]
            rows.append((k, s, p, cin, cout, h, h, N, best, best_plain))
            report.append(f"// N={N:3d} {name:9s} {cin:4d}->{cout:4d} k{k} {h:3d}x{h:<3d}: best {best} {best_us:8.1f} us "
                          f"{flop / best_us / 1e6:6.1f} TFLOP/s; worst {worst} {worst_us:8.1f} us ({worst_us / best_us:.2f}x)")
            print(report[-1], flush=True)
            del x, w, b, out
    kept = []
    if args.pooled_only:
        with open(args.out) as f:
            kept = [ln for ln in f.read().splitlines()[2:] if ln and " pool" not in ln and not ln.startswith("{1, 1, -1,")]
    with open(args.out, "w") as f:
        f.write("// Generated by paper_1611_07151_amd/tune.py on an MI355X: fastest tiling per layer shape and batch.\n")
        f.write("// {K, S, P, Cin, Cout, H, W, N, fastest tiling, fastest tiling that needs no scratch}\n")
        for line in [ln for ln in kept if ln.startswith("//")] + report:
            f.write(line + "\n")
        for line in [ln for ln in kept if not ln.startswith("//")]:
            f.write(line + "\n")
        for r in rows:
            f.write("{%d, %d, %d, %d, %d, %d, %d, %d, \"%s\", \"%s\"},\n" % r)
    print("wrote", args.out)
    return 0


if __name__ == "__main__":
    sys.exit(main())
