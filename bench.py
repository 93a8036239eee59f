#!/usr/bin/env python3
"""Benchmark: FP16 conv-forward throughput on the VGG-16-shaped stack at N=1.

A step is one pass of the whole hot path: the thirteen 3x3 convolution layers
(bias + ReLU fused), each launched through the C ABI on its own seeded synthetic
input already resident in HBM.  Prints ONE JSON line (see the keys below).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch N] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F16 = 2516.6e12     # MI355X dense FP16 MFMA FLOP/s
PEAK_HBM = 8.0e12             # MI355X HBM3E B/s

# (config, batch, entry, path, variant) -> HBM bytes per launch of the dominant kernel, from
# the rocprofv3 --pmc summaries under profiles/ (each states its calibration copy and commands)
TRAFFIC_BYTES_PER_LAUNCH = {
    # mean over the kernel's launches of a step: FETCH_SIZE KiB x 2.0 (copy calibration) + WRITE_SIZE KiB x 1.0
    # N=1: conv5..conv8 (three launches of grid 224, one of grid 112)
    ("vgg16", 1, "packed", "igemm", 82): int((2.0 * (3 * 5049.2 + 8712.0) / 4 + (3 * 1696.0 + 784.0) / 4) * 1024),
    # N=16: conv2 (grid 3136) and conv8..conv10 (grid 512)
    ("vgg16", 16, "packed", "igemm", 12): int((2.0 * (50960.9 + 3 * 20712.3) / 4 + (100876.7 + 3 * 12544.5) / 4) * 1024),
    # N=16: conv3, conv4 (grid 448) and conv5..conv7 (grid 256)
    ("vgg16", 16, "packed", "igemm", 0): int((2.0 * (2 * 20920.2 + 3 * 14477.3) / 5 + (2 * 52931.6 + 3 * 29106.3) / 5) * 1024),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=1, help="images per layer call (headline: 1)")
    ap.add_argument("--config", default="vgg16", help="workload table (headline: vgg16)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--entry", default="packed", choices=["packed", "ws", "plain"],
                    help="C entry point: hgc_conv2d_forward_packed (weights re-laid out once, before "
                         "timing, like a model load), hgc_conv2d_forward_ws or hgc_conv2d_forward")
    ap.add_argument("--tune", action="store_true",
                    help="after the headline measurement (launch shapes from the cost model), also run "
                         "hgc_conv2d_tune per layer (set-up-time measurement of the launch shapes) and time "
                         "the stack again; reported beside the headline")
    ap.add_argument("--per-layer", action="store_true", help="print a per-layer table to stderr")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also run a device-to-device copy of this many MiB ten times (a known-size "
                         "kernel that scales the HBM byte counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_1901_00858_amd as hgc
    from workloads import CONFIGS, layer_seed, make_tensors

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    hgc.load()
    dev = torch.device("cuda:0")
    layers = CONFIGS[args.config](args.batch)

    # ---- inputs resident in HBM before any timing ----
    host, bufs = [], []
    for i, L in enumerate(layers):
        x, w, b = make_tensors(L, seed=layer_seed(args.config, i))
        host.append((x, w, b))
        xd, wd, bd = (torch.from_numpy(a).to(dev) for a in (x, w, b))
        y = torch.empty(L.y_shape, dtype=torch.float16, device=dev)
        # the advertised size, or 32 MiB so that the tuning step may also try deeper reduction splits
        need = 0 if args.entry == "plain" else max(hgc.conv2d_workspace_size(L), 32 << 20)
        ws = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
        wp = hgc.conv2d_pack_weights(L, wd)          # one-time re-layout, outside every timed region
        bufs.append((hgc.ConvDesc.make(L), xd, wd, bd, y, ws, need, wp))
    stream = torch.cuda.current_stream(dev)
    sh = stream.cuda_stream
    if args.calibrate_copy:
        src = torch.ones(args.calibrate_copy << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()

    def launch(i, entry=args.entry):
        d, xd, wd, bd, y, ws, need, wp = bufs[i]
        if entry == "plain":
            st = hgc.forward_raw(d, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(), sh)
        elif entry == "ws":
            st = hgc.forward_ws_raw(d, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), y.data_ptr(),
                                    ws.data_ptr(), need, sh)
        else:
            st = hgc.forward_packed_raw(d, xd.data_ptr(), wp.data_ptr(), bd.data_ptr(), y.data_ptr(),
                                        ws.data_ptr(), need, sh)
        if st != 0:
            raise hgc.HgcError(st, layers[i].name)

    def timed(entry, steps, warmup):
        for _ in range(warmup):
            for i in range(len(layers)):
                launch(i, entry)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            for i in range(len(layers)):
                launch(i, entry)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    # bring the clocks up before anything is timed: an idle GPU needs some hundred
    # milliseconds of load to reach its working frequency, far more than W short steps
    t_spin = time.perf_counter()
    while time.perf_counter() - t_spin < 0.3:
        for i in range(len(layers)):
            launch(i)
        torch.cuda.synchronize()
    ms_per_step = timed(args.entry, args.steps, args.warmup)
    # the same stack through the entry point that takes the caller's weight layout
    other = "ws" if args.entry == "packed" else None
    ms_other = timed(other, max(1, args.steps // 4), max(1, args.warmup // 4)) if other else None
    flops_step = sum(L.flops for L in layers)
    bytes_step = sum(L.bytes for L in layers)
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12

    # ---- per-launch device time: an instrumented pass (the timed region above carries no events) runs
    # every layer `reps` times back to back between one pair of HIP events on the launch stream; the
    # average is the launch's duration including the dispatch gap to the next launch, as in the timed
    # chain.  (An event pair around each single launch adds the events' own gaps: two of them for a layer
    # with a split reduction, which is two kernels.) ----
    reps = max(5, min(50, args.steps))
    per_layer = []
    for i, L in enumerate(layers):
        launch(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            launch(i)
        e1.record(stream)
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        plan = hgc.conv2d_plan(L, args.entry != "plain", args.entry == "packed").as_dict()
        per_layer.append({
            "layer": L.name, "path": plan["path_name"], "variant": plan["variant"],
            "tile": [plan["tile_m"], plan["tile_h"], plan["tile_w"]], "split_k": plan["split_k"],
            "grid": plan["grid"], "us": us, "tflops": L.flops / us / 1e6, "gbs": L.bytes / us / 1e3,
            "flops": L.flops, "bytes": L.bytes,
        })
    # the dominant kernel: the instantiation whose launches take the largest share of a step
    groups = {}
    for r in per_layer:
        g = groups.setdefault((r["path"], r["variant"]), {"us": 0.0, "flops": 0, "bytes": 0, "n": 0, "layers": []})
        g["us"] += r["us"]; g["flops"] += r["flops"]; g["bytes"] += r["bytes"]; g["n"] += 1
        g["layers"].append(r["layer"])
    key, dom = max(groups.items(), key=lambda kv: kv[1]["us"])
    mfma_bound = (dom["flops"] / PEAK_MFMA_F16) >= (dom["bytes"] / PEAK_HBM)
    # HBM bytes per launch from the committed rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE scaled by
    # a plain copy of known size); see profiles/.  None when no such run covers this kernel/workload.
    traffic = TRAFFIC_BYTES_PER_LAUNCH.get((args.config, args.batch, args.entry, key[0], key[1]))
    if mfma_bound:
        achieved = dom["flops"] / dom["us"] / 1e6          # algorithmic TFLOP/s over its launches
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_F16 / 1e12, "unit": "TFLOP/s",
                "frac": achieved / (PEAK_MFMA_F16 / 1e12), "traffic": traffic}
    else:
        achieved = dom["bytes"] / dom["us"] / 1e3          # algorithmic GB/s over its launches
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                "frac": achieved / (PEAK_HBM / 1e9), "traffic": traffic}
    kname = hgc.igemm_variant_name(key[1], args.entry == "packed") if key[0].startswith("igemm") else key[0]
    roof.update({"kernel": kname + (", true>" if key[0] == "igemm_splitk" else ", false>" if key[0] == "igemm" else ""),
                 "layers": dom["layers"], "launches_per_step": dom["n"],
                 "avg_launch_us": dom["us"] / dom["n"],
                 "algorithmic_flops_per_launch": dom["flops"] / dom["n"],
                 "algorithmic_bytes_per_launch": dom["bytes"] / dom["n"],
                 "sum_layer_us": sum(r["us"] for r in per_layer)})

    if args.per_layer:
        for r in per_layer:
            print("%-12s %-13s v%-2d tile %-14s split %-2d grid %-5d %9.2f us %8.1f TFLOP/s %8.1f GB/s" % (
                r["layer"], r["path"], r["variant"], r["tile"], r["split_k"], r["grid"], r["us"],
                r["tflops"], r["gbs"]), file=sys.stderr)

    ms_tuned, tuned_layers = None, 0
    if args.tune and args.entry != "plain":   # after the roofline pass, which describes the headline shapes
        # launch shapes measured once per layer, outside every timed region, and the stack timed again
        for i, L in enumerate(layers):
            d, xd, wd, bd, y, ws, need, wp = bufs[i]
            before = hgc.conv2d_plan(L, True, args.entry == "packed").as_dict()
            st = hgc.tune_raw(d, xd.data_ptr(), (wp if args.entry == "packed" else wd).data_ptr(), bd.data_ptr(),
                              y.data_ptr(), ws.data_ptr(), need, args.entry == "packed", sh)
            if st != 0:
                raise hgc.HgcError(st, "tune " + L.name)
            tuned_layers += before != hgc.conv2d_plan(L, True, args.entry == "packed").as_dict()
        torch.cuda.synchronize()
        ms_tuned = timed(args.entry, args.steps, args.warmup)

    # ---- the classifier's inner-product layers (the next row after the convolution stack): HBM-bound,
    # reported beside the headline, never part of `value` ----
    fc_report = None
    fc_shapes = {"vgg16": [("fc6", 25088, 4096), ("fc7", 4096, 4096), ("fc8", 4096, 1000)],
                 "alexnet": [("fc6", 9216, 4096), ("fc7", 4096, 4096), ("fc8", 4096, 1000)]}.get(args.config)
    if fc_shapes:
        from workloads import uniform01, normal01
        fc_report = []
        for name, K, M in fc_shapes:
            Nb = args.batch
            xh = (2.0 * uniform01(7, 0, Nb * K) - 1.0).astype(np.float16).reshape(Nb, K)
            wh = (normal01(7, 1, M * K) * np.sqrt(2.0 / K)).astype(np.float16).reshape(M, K)
            bh = (0.2 * uniform01(7, 2, M) - 0.1).astype(np.float16)
            xd, wd, bd = (torch.from_numpy(a).to(dev) for a in (xh, wh, bh))
            yd = torch.empty((Nb, M), dtype=torch.float16, device=dev)
            d = hgc.InnerProductDesc(Nb, K, M, 1, 1)
            call = lambda: hgc.inner_product_forward_raw(d, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), yd.data_ptr(), sh)
            for _ in range(5):
                assert call() == 0
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(20):
                call()
            e1.record(stream)
            e1.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 20
            nbytes = 2 * (M * K + Nb * K + M + Nb * M)
            fc_report.append({"layer": name, "N": Nb, "K": K, "M": M, "us": us, "GB/s": nbytes / us / 1e3,
                              "frac_of_hbm_peak": nbytes / us / 1e3 / (PEAK_HBM / 1e9),
                              "algorithmic_bytes": nbytes})

    # ---- batch-norm layers at the shapes of this stack's feature maps (the row after the inner product):
    # HBM-bound, reported beside the headline, never part of `value`.  Algorithmic bytes: x read for the
    # statistics, read again for the output, y written (6 B per value); 4 B per value with stored statistics ----
    bn_shapes = {"vgg16": [(64, 224), (128, 112), (256, 56), (512, 28), (512, 14)],
                 "resnet50": [(64, 112), (256, 56), (512, 28), (1024, 14), (2048, 7)],
                 "mobilenet_v1": [(32, 112), (128, 56), (256, 28), (512, 14), (1024, 7)]}.get(args.config)
    bn_report = None
    if bn_shapes:
        from workloads import normal01
        bn_report = []
        for C, S in bn_shapes:
            Nb = args.batch
            n = Nb * C * S * S
            xh = (0.5 + 1.5 * normal01(9, 0, n)).astype(np.float16).reshape(Nb, C, S, S)
            xd = torch.from_numpy(xh).to(dev)
            yd = torch.empty_like(xd)
            gd = torch.ones(C, dtype=torch.float32, device=dev)
            bd = torch.zeros(C, dtype=torch.float32, device=dev)
            md = torch.zeros(C, dtype=torch.float32, device=dev)
            vd = torch.ones(C, dtype=torch.float32, device=dev)
            row = {"C": C, "H": S, "W": S, "N": Nb}
            for mode, glob, per in (("batch_statistics", 0, 6), ("stored_statistics", 1, 4)):
                d = hgc.BatchNormDesc(Nb, C, S, S, glob, 1, 1, 1e-5, 1.0)
                need = hgc.batch_norm_workspace_size(d)
                wsb = torch.empty(need, dtype=torch.uint8, device=dev)
                call = lambda: hgc.batch_norm_forward_raw(d, xd.data_ptr(), md.data_ptr(), vd.data_ptr(), gd.data_ptr(),
                                                          bd.data_ptr(), yd.data_ptr(), wsb.data_ptr(), need, sh)
                for _ in range(5):
                    assert call() == 0
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(20):
                    call()
                e1.record(stream)
                e1.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 20
                row[mode] = {"us": us, "GB/s": per * n / us / 1e3, "frac_of_hbm_peak": per * n / us / 1e3 / (PEAK_HBM / 1e9),
                             "algorithmic_bytes": per * n}
                md.zero_(); vd.fill_(1.0)
            bn_report.append(row)

    # ---- the whole VGG-16-shaped forward pass as one chain (the row after batch norm): the 13 convolutions of
    # the headline stack feeding each other through five 2x2 max-poolings, then fc6, fc7, fc8; every layer
    # reads the previous layer's output in HBM.  Reported beside the headline, never part of `value` ----
    chain = None
    if args.config == "vgg16" and args.entry == "packed":
        from workloads import uniform01, normal01
        pool_after = {1, 3, 6, 9, 12}                      # conv2, conv4, conv7, conv10, conv13
        Nb = args.batch
        steps_c = []                                      # (kind, descriptor, argument pointers..., output tensor)
        cur = bufs[0][1]                                  # the first layer's own input
        keep = []
        for i, L in enumerate(layers):
            d, _xd, _wd, bd, _y, ws, need, wp = bufs[i]
            yo = torch.empty((Nb, L.M, L.H, L.W), dtype=torch.float16, device=dev)
            steps_c.append(("conv", d, cur, wp, bd, yo, ws, need))
            cur = yo
            if i in pool_after:
                pd = hgc.MaxPoolDesc(Nb, L.M, L.H, L.W, 2, 2, 0)
                po = torch.empty((Nb, L.M, L.H // 2, L.W // 2), dtype=torch.float16, device=dev)
                steps_c.append(("pool", pd, cur, po))
                cur = po
        K = cur.numel() // Nb
        for name, M, relu in (("fc6", 4096, 1), ("fc7", 4096, 1), ("fc8", 1000, 0)):
            wh = (normal01(8, len(keep), M * K) * np.sqrt(2.0 / K)).astype(np.float16).reshape(M, K)
            bh = (0.2 * uniform01(8, 100 + len(keep), M) - 0.1).astype(np.float16)
            wd2, bd2 = torch.from_numpy(wh).to(dev), torch.from_numpy(bh).to(dev)
            keep.append((wd2, bd2))
            yo = torch.empty((Nb, M), dtype=torch.float16, device=dev)
            steps_c.append(("fc", hgc.InnerProductDesc(Nb, K, M, 1, relu), cur, wd2, bd2, yo))
            cur, K = yo, M

        def forward_chain():
            for st in steps_c:
                if st[0] == "conv":
                    _, d, xi, wp, bd, yo, ws, need = st
                    rc = hgc.forward_packed_raw(d, xi.data_ptr(), wp.data_ptr(), bd.data_ptr(), yo.data_ptr(),
                                                ws.data_ptr(), need, sh)
                elif st[0] == "pool":
                    rc = hgc.max_pool_forward_raw(st[1], st[2].data_ptr(), st[3].data_ptr(), sh)
                else:
                    _, d, xi, w2, b2, yo = st
                    rc = hgc.inner_product_forward_raw(d, xi.data_ptr(), w2.data_ptr(), b2.data_ptr(), yo.data_ptr(), sh)
                if rc != 0:
                    raise hgc.HgcError(rc, "chain " + st[0])

        for _ in range(max(3, args.warmup // 2)):
            forward_chain()
        torch.cuda.synchronize()
        csteps = max(5, args.steps // 2)
        t0 = time.perf_counter()
        for _ in range(csteps):
            forward_chain()
        torch.cuda.synchronize()
        ms_chain = (time.perf_counter() - t0) * 1e3 / csteps
        out_ok = bool(torch.isfinite(cur.float()).all().item())
        chain = {"what": "VGG-16-shaped forward pass: 13 conv (bias+ReLU) + 5 max-pool 2x2/2 + fc6, fc7 (ReLU), fc8, chained in HBM",
                 "calls_per_step": len(steps_c), "steps": csteps, "ms_per_step": ms_chain, "ms_per_image": ms_chain / Nb,
                 "images_per_s": Nb / (ms_chain * 1e-3), "output_finite": out_ok}

    # ---- the oracle, as it stands, timed on the host cores (a reported baseline) ----
    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.build()
        sample = [i for i, L in enumerate(layers)] if args.batch == 1 else [len(layers) - 1]
        t = time.perf_counter()
        fl = 0
        passes = 0
        while True:                                   # whole passes until about ten seconds of CPU work are in
            for i in sample:
                x, w, b = host[i]
                oracle.conv2d_forward(layers[i].desc(), x, w, b)
                fl += layers[i].flops
            passes += 1
            dt = time.perf_counter() - t
            if dt >= 10.0 or passes >= 50:
                break
        cpu = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%d pass%s over %d of the %d layers at N=%d (%.2f GFLOP, %.1f s)" % (
                   passes, "" if passes == 1 else "es", len(sample), len(layers), args.batch, fl / 1e9, dt),
               "ms_per_image": dt * 1e3 / passes / args.batch if len(sample) == len(layers) else None}

    out = {
        "metric": "FP16 conv-forward TFLOP/s, VGG-16-shaped 13-layer stack",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_image": ms_per_step / args.batch,
        "pct_mfma_peak": 100.0 * tflops / (PEAK_MFMA_F16 / 1e12),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 (fp32 accumulate)", "data": "synthetic",
        "config": {"workload": "%s conv stack, N=%d, 3x3 s1 p1, bias+ReLU, %d layers, %.2f GFLOP, %.1f MB" % (
            args.config, args.batch, len(layers), flops_step / 1e9, bytes_step / 1e6),
            "entry": {"packed": "hgc_conv2d_forward_packed (weights packed once before timing)",
                      "ws": "hgc_conv2d_forward_ws", "plain": "hgc_conv2d_forward"}[args.entry]},
        "tuned_launch_shapes": None if ms_tuned is None else {
            "entry": "hgc_conv2d_tune per layer before timing", "layers_changed": tuned_layers,
            "ms_per_step": ms_tuned, "value": flops_step / (ms_tuned * 1e-3) / 1e12, "unit": "TFLOP/s"},
        "caller_layout_weights": None if ms_other is None else {
            "entry": "hgc_conv2d_forward_ws", "ms_per_step": ms_other,
            "value": flops_step / (ms_other * 1e-3) / 1e12, "unit": "TFLOP/s"},
        "inner_product_layers": fc_report,
        "batch_norm_layers": bn_report,
        "full_forward": chain,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
