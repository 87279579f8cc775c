"""Benchmark of the fixed-point inference hot path on one MI355X.

One step = one forward pass of the whole fixed-point ResNet-50 (stride on the 3x3 of the
bottleneck) over a batch of 256 seeded synthetic 224x224x3 images that already sit in HBM:
53 dense layers + FC on the int8 matrix cores with the shift/clip epilogue, max pool,
global pool.  Prints ONE JSON line.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 matrix peak, TOP/s
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E peak, GB/s

TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "resnet50_b256_hbm_traffic.md")
KERNEL_SOURCES = os.path.join(ROOT, "paper_2202_05239_amd", "csrc")


def kernel_source_hash():
    """Short hash over the kernel sources: ties a committed counter profile to the code it measured."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(KERNEL_SOURCES)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(KERNEL_SOURCES, name), "rb").read())
    return h.hexdigest()[:16]


def traffic_from_profile():
    """HBM bytes per launch of every kernel of the ResNet-50 batch-256 forward, from the committed
    rocprofv3 FETCH_SIZE / WRITE_SIZE summary (counters cannot be read from inside this process).
    Returns ({bench kernel name: MB per launch}, the kernel-source hash the profile was taken at)."""
    table, src = {}, None
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("kernel sources:"):
                src = line.split(":", 1)[1].strip()
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 6 and cells[0].startswith("`") and cells[-1].replace(".", "", 1).isdigit():
                table[cells[0].strip("`")] = float(cells[-1])
    except OSError:
        pass
    return table, src


def cpu_baseline(net, x, threads, images):
    """The CPU oracle as it stands, on `images` images of the same workload, one image per
    host thread (the C code itself is single-threaded)."""
    import numpy as np
    from oracle import ref
    xs = np.ascontiguousarray(x[:images])
    t0 = time.perf_counter()
    ref.run_network_parallel(net, xs, threads)
    dt = time.perf_counter() - t0
    return {"value": images / dt, "unit": "images/s", "cores": threads, "kind": "oracle",
            "sample": "%d of the %d images of the batch, full 224x224 ResNet-50 forward, one image per "
                      "host thread, %.1f s wall" % (images, x.shape[0], dt)}


def layer_rows(f8, net, chain, layer_ms, B):
    """Per-layer table: time, algorithmic ops and bytes, fractions of both rooflines."""
    rows = []
    for i, (L, ms) in enumerate(zip(net.layers, layer_ms)):
        kname, ops, nbytes = chain.layer_info(i, B)
        t = max(ms, 1e-6) * 1e-3                    # layers absorbed into a fused block take no time
        tops, gbs = ops / t / 1e12, nbytes / t / 1e9
        t_mfma, t_hbm = ops / (PEAK_INT8_TOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
        rows.append({"layer": L.name, "kernel": kname, "us": ms * 1e3, "ops": ops, "bytes": nbytes, "TOPS": tops,
                     "pct_mfma_peak": 100 * tops / PEAK_INT8_TOPS, "alg_GBs": gbs,
                     "pct_hbm_peak": 100 * gbs / PEAK_HBM_GBS,
                     "binds": "mfma" if (L.op == "conv" and t_mfma > t_hbm) else "hbm",
                     "pct_of_roofline": 100 * max(t_mfma if L.op == "conv" else 0.0, t_hbm) / t})
    return rows


def single_layer_figures(torch, f8, wl, repeats):
    """The two single-layer figures of the headline metric, timed with HIP events on the
    launch stream through the same chain runner: the 3x3 dense layer of configs[1] (TOP/s
    against the int8 matrix peak) and the depthwise layer of configs[2] (algorithmic GB/s
    against the HBM peak), plus the streaming copy as the yardstick of what HBM gives."""
    out = {}
    x1, L1 = wl.config1()
    net1 = wl.Net(name="config1", in_hw=L1.in_hw, in_c=L1.Cin, x_type=L1.x_type, fl_x=L1.fl_x, layers=[L1])
    x2, net2 = wl.config2(with_residual=True)
    for key, x, net in (("configs[1]", x1, net1), ("configs[2]", x2, net2)):
        B = x.shape[0]
        xt = torch.from_numpy(x).to("cuda")
        chain = f8.Chain(net).prepare(B)
        y = torch.empty((B,) + chain.out_shape, dtype=chain.out_dtype, device="cuda")
        chain.run(xt, y)
        ms = chain.profile(xt, y, repeats=repeats)
        for r in layer_rows(f8, net, chain, ms, B):
            out["%s %s" % (key, r["layer"])] = {k: r[k] for k in
                                                ("kernel", "us", "TOPS", "pct_mfma_peak", "alg_GBs", "pct_hbm_peak", "binds")}
        chain.close()
    # a layer of a single tile, timed the same way: what one dependent launch costs on its own
    import numpy as np
    rng = np.random.default_rng(7)
    nb = wl._NetBuilder("one_tile", rng, 8, 64, "u8", 5, (5, 9), (2, 6), False)
    nb.conv("conv1x1", 0, 64, 1, 1, 0)
    xt = torch.from_numpy(wl.draw_u8(rng, (1, 8, 8, 64))).to("cuda")
    chain = f8.Chain(nb.net).prepare(1)
    y = torch.empty((1,) + chain.out_shape, dtype=chain.out_dtype, device="cuda")
    chain.run(xt, y)
    out["one-tile layer (floor of a launch in this timing)"] = {"us": chain.profile(xt, y, repeats=repeats)[0] * 1e3}
    chain.close()
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    f8.f8_copy_bytes(a, b)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        f8.f8_copy_bytes(a, b)
    e1.record()
    torch.cuda.synchronize()
    out["copy 1 GiB"] = {"GBs_read_plus_write": 2.0 * n * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9}
    # register-only loop of the int8 matrix instruction: the practical ceiling of the matrix cores
    sink = torch.empty(f8.F8_YARDSTICK_SINK_INTS, dtype=torch.int32, device="cuda")
    f8.f8_mfma_i8_yardstick(sink, 2000)
    e0.record()
    ops = sum(f8.f8_mfma_i8_yardstick(sink, 20000) for _ in range(5))
    e1.record()
    torch.cuda.synchronize()
    out["mfma i8 register-only loop"] = {"TOPS": ops / (e0.elapsed_time(e1) * 1e-3) / 1e12}
    # the same loop on operands whose every bit is pseudo-random, as real tensors' are
    f8.f8_mfma_i8_yardstick_operands(sink, 2000, 1)
    e0.record()
    ops = sum(f8.f8_mfma_i8_yardstick_operands(sink, 20000, 1 + k) for k in range(5))
    e1.record()
    torch.cuda.synchronize()
    out["mfma i8 register-only loop, random operand bytes"] = {"TOPS": ops / (e0.elapsed_time(e1) * 1e-3) / 1e12}
    return out


def copy_calibration():
    """Three launches of the plain copy kernel over 1 GiB: the known-size reference for
    the FETCH_SIZE / WRITE_SIZE counters."""
    import torch
    from paper_2202_05239_amd import binding as f8
    n = 1 << 30
    a = torch.zeros(n, dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        f8.f8_copy_bytes(a, b)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_per_launch": n}))


def mfma_calibration():
    """Three launches of the register-only int8 matrix-instruction loop: the known-size reference
    for the matrix-core counters (every SIMD issues matrix instructions back to back)."""
    import torch
    from paper_2202_05239_amd import binding as f8
    sink = torch.empty(f8.F8_YARDSTICK_SINK_INTS, dtype=torch.int32, device="cuda")
    ops = [f8.f8_mfma_i8_yardstick(sink, 20000) for _ in range(3)]
    torch.cuda.synchronize()
    print(json.dumps({"mfma_ops_per_launch": ops[0]}))


def quant_tools_figures(repeats=10):
    """Throughput of the steps upstream of the integer layers on a 1 GiB float32 tensor
    (2^28 elements ~ N(0, 1)) and of the folding of a 2048 x 4608 Conv-BN block, timed with
    HIP events on the launch stream; algorithmic bytes = every input element read once, every
    output element written once."""
    import torch
    from paper_2202_05239_amd import binding as f8
    L = f8.lib()
    n = 1 << 28
    x = torch.randn(n, device="cuda")
    y = torch.empty_like(x)
    q = torch.empty(n, dtype=torch.uint8, device="cuda")
    work = torch.empty(f8.F8_STATS_WORK_DOUBLES + 2 * 2048, dtype=torch.float64, device="cuda")
    out = torch.empty(3, dtype=torch.float64, device="cuda")
    stats = torch.empty(24, dtype=torch.uint8, device="cuda")
    cout, k = 2048, 4608
    w = x[:cout * k].view(cout, k)
    wq = torch.empty((cout, k), dtype=torch.int8, device="cuda")
    bq = torch.empty(cout, dtype=torch.int32, device="cuda")
    g, beta, mu, sg = (torch.rand(cout, device="cuda") + 0.5 for _ in range(4))
    s = f8._stream()
    desc = f8.f8_fold_desc(cout, k, 0.3, 0.2, 4, -1)
    rows = [
        ("fix_quant_f32 (Eq. 2/9)", 8 * n, lambda: f8.f8_fix_quant_f32(x, 5, True, out=y)),
        ("fix_quant_code (Eq. 2/9)", 5 * n, lambda: f8.f8_fix_quant_code(x, 5, False, out=q)),
        ("pact_f32 (Eq. 3)", 8 * n, lambda: f8.f8_pact_f32(x, 4.7, out=y)),
        ("pact_fix_f32 (Eq. 4)", 8 * n, lambda: f8.f8_pact_fix_f32(x, 4.7, 5, out=y)),
        ("tensor_stats_f32 (Eq. 1)", 4 * n, lambda: L.f8_tensor_stats_f32(f8._ptr(x), n, f8._ptr(stats), f8._ptr(work), s)),
        ("quant_error_f32 (toy experiment)", 4 * n, lambda: f8.f8_quant_error_f32(x, 5, True, out=out, work=work)),
        ("fold_conv_bn 2048x4608 (Eq. 6, FL_w by Eq. 1)", 9 * cout * k + 24 * cout,
         lambda: L.f8_fold_conv_bn(f8._ptr(w), f8._ptr(g), f8._ptr(beta), f8._ptr(mu), f8._ptr(sg), ctypes.byref(desc),
                                   f8._ptr(wq), f8._ptr(bq), f8._ptr(stats), f8._ptr(work), s)),
    ]
    res = {}
    for name, nbytes, fn in rows:
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(repeats):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / repeats
        res[name] = {"us": us, "alg_MB": nbytes / 1e6, "alg_GBs": nbytes / us / 1e3,
                     "pct_hbm_peak": 100 * nbytes / us / 1e3 / PEAK_HBM_GBS}
    print(json.dumps({"quant_tools": res}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--net", default="resnet50", choices=["resnet50", "resnet18", "mobilenetv2", "mobilenetv1", "resnet50_private_fl"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch the chain eagerly instead of replaying a HIP graph")
    ap.add_argument("--layers", default="", help="write the per-layer table (JSON) to this file")
    ap.add_argument("--fusion", action="store_true", help="run inverted-residual blocks as one fused kernel")
    ap.add_argument("--streams", type=int, default=2, choices=[1, 2],
                    help="2: the two halves of the batch side by side on two streams inside every step (default); 1: one stream")
    ap.add_argument("--no-single-layer", action="store_true", help="skip the configs[1] / configs[2] layer figures")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run the plain copy kernel on 1 GiB (reference for the traffic counters)")
    ap.add_argument("--mfma-calibration", action="store_true",
                    help="only run the register-only matrix-instruction loop (reference for the matrix-core counters)")
    ap.add_argument("--quant-tools", action="store_true",
                    help="only time the steps upstream of the integer layers (quantisers, statistics, folding)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
              "(the path shards by batch: images are independent, no communication)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.copy_calibration:
        copy_calibration()
        return
    if args.mfma_calibration:
        mfma_calibration()
        return
    if args.quant_tools:
        quant_tools_figures()
        return

    import torch
    from paper_2202_05239_amd import binding as f8
    from paper_2202_05239_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    f8.lib()     # fails loudly if the HIP library is missing

    if args.net == "resnet50":
        x, net = wl.config4(batch=args.batch)
    elif args.net == "resnet18":
        x, net = wl.config3(batch=args.batch)
    elif args.net == "mobilenetv2":
        x, net = wl.mobilenet_v2_forward(batch=args.batch)
    elif args.net == "resnet50_private_fl":
        x, net = wl.resnet50_private_fl(batch=args.batch)
    else:
        x, net = wl.mobilenet_v1_forward(batch=args.batch)
    B = x.shape[0]
    xt = torch.from_numpy(x).to("cuda")
    chain = f8.Chain(net, fusion=args.fusion, streams=args.streams).prepare(B)
    out = torch.empty((B,) + chain.out_shape, dtype=chain.out_dtype, device="cuda")

    # One step = one replay of the captured chain (all layers, nothing skipped); the eager
    # result is kept to check that the replays reproduce it bit for bit.
    chain.run(xt, out)
    torch.cuda.synchronize()
    eager = out.clone()
    step = chain.run
    if not args.no_graph:
        graph = chain.capture(xt, out)
        step = lambda *_: graph.replay()
    for _ in range(args.warmup):
        step(xt, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(xt, out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same steps once more with an event between them (on the stream they run on): per-step
    # device times for the median; `value` above comes from the host clock around all K steps
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        step(xt, out)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    median_ms = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
    if not torch.equal(out, eager):
        print("bench.py: graph replay differs from the eager run", file=sys.stderr)
        sys.exit(4)
    ms_per_step = dt / args.steps * 1e3
    images_per_s = B / (dt / args.steps)

    # Per-kernel device time of the same steps, HIP events on the launch stream.
    layer_ms = chain.profile(xt, out, repeats=max(1, args.steps))
    rows, by_kernel = layer_rows(f8, net, chain, layer_ms, B), {}
    for r in rows:
        k = by_kernel.setdefault(r["kernel"], {"ms": 0.0, "ops": 0.0, "bytes": 0.0, "launches": 0})
        k["ms"] += r["us"] * 1e-3; k["ops"] += r["ops"]; k["bytes"] += r["bytes"]; k["launches"] += 1
    dom = max(by_kernel, key=lambda n: by_kernel[n]["ms"])
    d = by_kernel[dom]
    t_m, t_h = d["ops"] / (PEAK_INT8_TOPS * 1e12), d["bytes"] / (PEAK_HBM_GBS * 1e9)
    if t_m >= t_h:
        ach = d["ops"] / (d["ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": ach / PEAK_INT8_TOPS}
    else:
        ach = d["bytes"] / (d["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}
    # counter traffic: only for the workload the committed profile covers, and only if the kernel
    # sources are the ones it was measured on (null otherwise, with the reason)
    table, profiled_src = traffic_from_profile()
    traffic, note = None, "no counter profile for this workload"
    if args.net == "resnet50" and B == 256:
        if profiled_src != kernel_source_hash():
            note = "profiles/resnet50_b256_hbm_traffic.md was measured on other kernel sources (%s)" % profiled_src
        elif dom not in table:
            note = "kernel not in profiles/resnet50_b256_hbm_traffic.md"
        else:
            traffic, note = table[dom], "profiles/resnet50_b256_hbm_traffic.md (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the copy kernel)"
    roof.update({"traffic": traffic * 1e6 if traffic is not None else None, "traffic_unit": "bytes per launch",
                 "traffic_source": note,
                 "alg_bytes_per_launch": d["bytes"] / d["launches"], "kernel": dom, "launches_per_step": d["launches"],
                 "avg_launch_us": d["ms"] * 1e3 / d["launches"],
                 "alg_ops_per_step": d["ops"], "alg_bytes_per_step": d["bytes"],
                 "sum_layer_ms": sum(layer_ms)})
    if args.layers:
        with open(args.layers, "w") as f:
            json.dump({"layers": rows, "kernels": by_kernel}, f, indent=1)

    total_ops = sum(2.0 * L.macs_per_image * B for L in net.layers)
    rec = {
        "metric": "images/s, fixed-point %s forward (int8 conv on MFMA + shift/clip epilogue), batch %d, 1 GPU"
                  % ({"resnet50": "ResNet-50", "resnet18": "ResNet-18", "mobilenetv2": "MobileNetV2", "mobilenetv1": "MobileNetV1",
                      "resnet50_private_fl": "ResNet-50 (two formats per block output)"}[args.net], B),
        "value": images_per_s, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "median_ms_per_step": median_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: full %s fixed-point forward, batch %d, 224x224x3, seeded FL per layer"
                               % ({"resnet50": "configs[4]", "resnet18": "configs[3]"}.get(args.net, "extra"),
                                  net.name, B),
                   "global_batch": B, "input": "224x224x3 int8", "layers": len(net.layers),
                   "streams_per_step": args.streams},
        "whole_net_TOPS": total_ops / (dt / args.steps) / 1e12,
        "roofline": roof,
    }
    if not args.no_single_layer:
        rec["single_layer"] = single_layer_figures(torch, f8, wl, repeats=50)
    if not args.no_cpu_baseline:
        threads = max(1, min(16, os.cpu_count() or 1, 8))
        rec["cpu_baseline"] = cpu_baseline(net, x, threads, threads)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
