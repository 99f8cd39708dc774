#!/usr/bin/env python3
"""Benchmark of the grouped-convolution hot path on one MI355X.

A step is one forward pass of the WRN-40-2-style CIFAR stack (every 3x3 conv
after the stem grouped, fp32, batch 64) for each g in {1, 2, 4, 8, 16}: five
layer chains, 195 convolution launches, run through gspc_run_layer_chain with
all tensors resident in HBM.  `value` is the Eq. 2 MAC count of the step
divided by its time.  Prints ONE JSON line.

Also reported on the same line:
  roofline     - for the kernel that takes the largest share of the step: its
                 algorithmic flops (or bytes) per launch over its average
                 launch duration, measured here with events on the launch
                 stream by running each of its layers back to back.
  roofline_direct - when that kernel instance is the Winograd one: the same object for the
                 direct-sum instance with the largest share (null otherwise).
  roofline_hbm - the same for the HBM-bound side of the path: the MobileNet-shaped
                 depthwise 3x3 layers at batch 256 over rotating buffers, dominant kernel.
  latency_ms   - batch-1 latency of the WRN-40-2-style and ResNet-34-shaped networks
                 for every g (the quantity of the paper's Tables II-III), recorded chains.
  cpu_baseline - the CPU oracle timed on the host cores: all cores on the same batch,
                 one thread on a smaller sample, and Algorithm 1 in its vectorised CPU
                 schedule ("the paper's method on the host").
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GROUPS = (1, 2, 4, 8, 16)
BATCH = 64
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def layer_flops_bytes(l):
    from paper_2006_09791_amd import workloads as wl
    ho, wo = wl.out_size(l.H, l.KH, l.stride, l.pad), wl.out_size(l.W, l.KW, l.stride, l.pad)
    macs = l.N * l.Cin * l.Cout * l.KH * l.KW * ho * wo // l.groups
    out_b = l.N * l.Cout * ho * wo * 4
    nbytes = l.N * l.Cin * l.H * l.W * 4 + l.Cout * (l.Cin // l.groups) * l.KH * l.KW * 4 + out_b
    if l.src2 >= 0:
        nbytes += out_b          # fused residual read
    return 2 * macs, nbytes


def _roofline_object(name, k, kernels):
    """Roofline object of one kernel instance: its summed algorithmic work over its summed event-timed
    duration, against the matrix-core peak (compute-bound layers) or the HBM peak."""
    traffic = None
    if os.path.exists(TRAFFIC_FILE):
        try:
            traffic = json.load(open(TRAFFIC_FILE)).get(name)
        except Exception:
            traffic = None
    if ("mfma" in name or "wino" in name) and k["compute_bound"]:
        ach = k["flops"] / k["time"] / 1e12
        roofline = {"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_F32_MFMA_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / PEAK_F32_MFMA_TFLOPS, 4)}
        if "wino" in name:
            # Eq. 2 counts the multiplications of the direct sum; the Winograd kernel executes 16/36 of them.
            # `achieved` and `frac` are the executed work against the matrix-core peak (a roofline fraction);
            # the Eq. 2 rate is an effective figure and is reported as such, without a fraction.
            roofline["algorithm"] = "winograd F(2x2,3x3): executes 16/36 of the Eq. 2 multiplications"
            roofline["eq2_effective_tflops"] = round(ach, 2)
            roofline["achieved"] = round(ach * 16.0 / 36.0, 2)
            roofline["frac"] = round(ach * 16.0 / 36.0 / PEAK_F32_MFMA_TFLOPS, 4)
    else:
        ach = k["bytes"] / k["time"] / 1e9
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4)}
    traffic_at = None
    if os.path.exists(TRAFFIC_FILE):
        try:
            traffic_at = json.load(open(TRAFFIC_FILE)).get("_measured_at")
        except Exception:
            pass
    roofline.update({"traffic": traffic, "traffic_measured_at": traffic_at,
                     "traffic_algorithmic": round(k["bytes"] / k["launches"]),
                     "kernel": name, "launches_per_step": k["launches"],
                     "avg_launch_us": round(k["time"] / k["launches"] * 1e6, 2),
                     "share_of_step": round(k["time"] / sum(v["time"] for v in kernels.values()), 3)})
    return roofline


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the roofline_hbm and latency_ms legs")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="first run a plain 256 MiB device copy three times: the known-size kernel "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    ap.add_argument("--sweep", choices=["wrn", "wrn_n256", "resnet_bf16", "depthwise", "blocks", "latency", "winograd", "mobilenetv2", "yardstick"],
                    help="instead of the headline step, time every layer of a configuration family "
                         "and print one JSON line with a row per layer")
    ap.add_argument("--fusion", action="store_true",
                    help="let the timed step fuse runs of grouped layers (one kernel per run); off by "
                         "default: with five chains in flight the separate small kernels overlap better")
    ap.add_argument("--serial", action="store_true",
                    help="run the five chains of a step one after the other on one stream")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); "
              "no multi-GPU path exists", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2006_09791_amd import binding as b
    from paper_2006_09791_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    b.load()                       # raises if libgspc.so is missing: no fallback
    # All work goes to one non-default stream (default priority): the chain
    # runner records its launches into HIP graphs only off the null stream.
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    b.gspc_set_stream()

    if args.traffic_probe:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)      # one elementwise kernel: reads and writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    if args.sweep:
        from paper_2006_09791_amd import layer_timing
        if args.sweep == "wrn":
            shapes = [s for g in GROUPS for s in wl.wrn_grouped_shapes(BATCH, g)]
            rows = layer_timing.time_layers(shapes, "f32")
        elif args.sweep == "yardstick":
            # A yardstick from outside this library, for context only: the vendor library's batched GEMM
            # (torch.bmm) on each layer's per-group contraction, [g][N*Hout*Wout][CPG*9] x [g][CPG*9][KPG], with the
            # im2col matrix given to it for free (forming it would move nine times the input).  Same flops as Eq. 2.
            rows = []
            legs = [("f32", [s for g in (1, 2, 4) for s in wl.wrn_grouped_shapes(BATCH, g)]),
                    ("bf16", [s for s in wl.resnet34_grouped_shapes(256, 2)])]
            b.gspc_set_winograd(0)   # like against like: the direct sum on both sides
            for dtype, shapes in legs:
                seen = []
                for s in shapes:
                    if s not in seen:
                        seen.append(s)
                ours = layer_timing.time_layers(seen, dtype, inner=6, reps=5)
                for s, r in zip(seen, ours):
                    ho, wo = b.gspc_output_dims(s.H, s.W, s.KH, s.KW, s.stride, s.pad)
                    P, K, KPG = s.N * ho * wo, (s.Cin // s.groups) * s.KH * s.KW, s.Cout // s.groups
                    td = torch.bfloat16 if dtype == "bf16" else torch.float32
                    A = torch.randn(s.groups, P, K, device=dev, dtype=td)
                    Bm = torch.randn(s.groups, K, KPG, device=dev, dtype=td)
                    out = torch.empty(s.groups, P, KPG, device=dev, dtype=td)
                    for _ in range(3):
                        torch.bmm(A, Bm, out=out)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    torch.cuda.synchronize()
                    e0.record()
                    for _ in range(20):
                        torch.bmm(A, Bm, out=out)
                    e1.record()
                    torch.cuda.synchronize()
                    us = e0.elapsed_time(e1) / 20 * 1e3
                    rows.append({"layer": r["layer"], "dtype": dtype, "kernel": r["kernel"], "us": r["us"], "tflops": r["tflops"],
                                 "gemm": f"{s.groups} x [{P} x {K}] x [{K} x {KPG}]", "library_gemm_us": round(us, 2),
                                 "library_gemm_tflops": round(2.0 * s.groups * P * K * KPG / us / 1e6, 2)})
                    del A, Bm, out
            b.gspc_set_winograd(None)
        elif args.sweep == "wrn_n256":
            # the compute-bound layers again at batch 256: steady-state matrix-core efficiency
            shapes = [s for g in (1, 2, 4) for s in wl.wrn_grouped_shapes(256, g) if s.stride == 1]
            shapes += [s for s in wl.wrn_grouped_shapes(1024, 1) if s.stride == 1]
            rows = layer_timing.time_layers(shapes, "f32", inner=4, reps=5)
        elif args.sweep == "latency":
            # whole-network latency at batch 1 (recorded chains replayed back to back)
            rows = []
            nets = [(f"wrn40x2-style g={g}", wl.wrn_chain(1, g), 2) for g in GROUPS]
            nets += [(f"resnet34-shaped g={g}", wl.resnet34_chain(1, g), 3) for g in (2, 4, 8, 16, 32)]
            nets += [(f"mobilenet-shaped {'G(N) depthwise' if g is None else 'g=' + str(g)}", wl.mobilenet_chain(1, g), 5)
                     for g in (2, 4, 8, 16, None)]
            nets += [(f"mobilenetv2-shaped {'G(N) depthwise' if g is None else 'g=' + str(g)}", wl.mobilenetv2_chain(1, g), 6)
                     for g in (2, 4, 8, 16, None)]
            nets += [(f"wrn40x2 pointwise form g={g}", wl.wrn_chain(1, g, pointwise=True), 7) for g in (2, 4, 8, 16)]
            nets += [(f"resnet34 pointwise form g={g}", wl.resnet34_chain(1, g, pointwise=True), 7) for g in (2, 4, 8, 16, 32)]
            nets += [(f"depthwise+pointwise C={C} {hw}x{hw} s{st}", wl.mobilenet_dw_chain(1, C, hw, st), 4)
                     for C, hw in wl.DEPTHWISE_CH_HW for st in (1, 2)]
            for name, ch, cfg in nets:
                weights = ch.make_weights(cfg)
                packed = [b.gspc_pack_weights(torch.from_numpy(w).to(dev), gg)
                          for w, gg in zip(weights, ch.weight_groups)]
                bufs = [torch.empty(max(n, 1), dtype=torch.float32, device=dev) for n in ch.buf_elems]
                bufs[0].copy_(torch.from_numpy(wl.make_input(ch.input_shape, 1)).reshape(-1))
                lc = b.LayerChain(ch.layers, packed, bufs)
                for _ in range(5):
                    b.gspc_run_layer_chain(lc)
                torch.cuda.synchronize()
                reps = 100
                ta = time.perf_counter()
                for _ in range(reps):
                    b.gspc_run_layer_chain(lc)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - ta) / reps * 1e3
                rows.append({"network": name, "layers": len(ch.layers), "mmacs": round(ch.macs() / 1e6, 2),
                             "latency_ms": round(ms, 4), "gmacs": round(ch.macs() / ms / 1e6, 1)})
        elif args.sweep == "winograd":
            # the stride-1 3x3 layers with at least 8 channels per group, direct and through
            # Winograd F(2x2, 3x3) (Section VI names grouped Winograd as the next step)
            rows = []
            for N in (64, 256):
                shapes = [s for g in (1, 2, 4) for s in wl.wrn_grouped_shapes(N, g) if s.stride == 1 and s.Cin // s.groups >= 8]
                shapes += [s for g in (2, 4, 8) for s in wl.resnet34_grouped_shapes(N, g) if s.stride == 1 and s.Cin // s.groups >= 8]
                b.gspc_set_winograd(0)
                direct = layer_timing.time_layers(shapes, "f32", inner=4, reps=5)
                b.gspc_set_winograd(1)
                wino = layer_timing.time_layers(shapes, "f32", inner=4, reps=5)
                b.gspc_set_winograd(None)
                auto = layer_timing.time_layers(shapes, "f32", inner=4, reps=5)
                for d, w, a in zip(direct, wino, auto):
                    rows.append({"layer": d["layer"], "direct_kernel": d["kernel"], "direct_us": d["us"],
                                 "direct_frac_mfma": d["frac_mfma"], "winograd_kernel": w["kernel"], "winograd_us": w["us"],
                                 "speedup": round(d["us"] / w["us"], 3), "default_kernel": a["kernel"], "default_us": a["us"]})
        elif args.sweep == "mobilenetv2":
            # the MobileNetV2-shaped network (Section IV-A) at batch 64, G(g) for g in {2,4,8,16} and the
            # depthwise original G(N): whole forward passes as recorded chains
            rows = []
            for g in (2, 4, 8, 16, None):
                ch = wl.mobilenetv2_chain(64, g)
                weights = ch.make_weights(6)
                packed = [b.gspc_pack_weights(torch.from_numpy(w).to(dev), gg)
                          for w, gg in zip(weights, ch.weight_groups)]
                bufs = [torch.empty(max(n, 1), dtype=torch.float32, device=dev) for n in ch.buf_elems]
                bufs[0].copy_(torch.from_numpy(wl.make_input(ch.input_shape, 1)).reshape(-1))
                lc = b.LayerChain(ch.layers, packed, bufs)
                for _ in range(3):
                    b.gspc_run_layer_chain(lc)
                torch.cuda.synchronize()
                reps = 20
                ta = time.perf_counter()
                for _ in range(reps):
                    b.gspc_run_layer_chain(lc)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - ta) / reps * 1e3
                rows.append({"network": f"mobilenetv2-shaped {'G(N) depthwise' if g is None else 'g=' + str(g)} N=64",
                             "layers": len(ch.layers), "gmacs_per_pass": round(ch.macs() / 1e9, 2),
                             "ms": round(ms, 3), "tmacs": round(ch.macs() / ms / 1e9, 1)})
                del lc, bufs, packed
        elif args.sweep == "blocks":
            # depthwise 3x3 + pointwise 1x1 blocks, as two kernels and with chain fusion
            rows = layer_timing.time_blocks(wl.depthwise_pairs(256), inner=8, reps=5)
        elif args.sweep == "resnet_bf16":
            # each layer twice: re-using one input and one output buffer (a working set of up to
            # 308 MB, of which the 256 MB last-level cache keeps a part), and over a rotation of three
            # buffer sets, so that every launch streams from and to HBM
            shapes = [s for g in (2, 8, 32) for s in wl.resnet34_grouped_shapes(256, g)]
            rows = layer_timing.time_layers(shapes, "bf16", inner=4, reps=5)
            cold = layer_timing.time_layers(shapes, "bf16", inner=6, reps=4, rotate=3)
            for r, c in zip(rows, cold):
                r["us_rotating"] = c["us"]
                r["gbs_rotating"] = c["gbs"]
                r["frac_hbm_rotating"] = c["frac_hbm"]
        else:
            # batched re-run of the MobileNet-shaped depthwise layers; buffer sets
            # rotate so that every launch streams from HBM rather than from cache
            shapes = [dw for dw, _ in wl.depthwise_pairs(256)]
            rows = layer_timing.time_layers(shapes, "f32", inner=8, reps=5, rotate=4)
        print(json.dumps({"sweep": args.sweep, "rows": rows}))
        return 0

    # ---- build the five chains, everything resident on the device ----------
    chains, lcs, keep = [], [], []
    for g in GROUPS:
        ch = wl.wrn_chain(BATCH, g)
        weights = ch.make_weights(2)
        packed = [b.gspc_pack_weights(torch.from_numpy(w).to(dev), gg)
                  for w, gg in zip(weights, ch.weight_groups)]
        bufs = [torch.empty(max(n, 1), dtype=torch.float32, device=dev) for n in ch.buf_elems]
        x0 = wl.make_input(ch.input_shape, wl.make_seed(2, 999, g))
        bufs[0].copy_(torch.from_numpy(x0).reshape(-1))
        chains.append(ch)
        lcs.append(b.LayerChain(ch.layers, packed, bufs))
        keep.append((packed, bufs))
    macs_step = sum(ch.macs() for ch in chains)

    # The five chains of a step are independent of each other, so each runs on
    # a stream of its own (all at default priority) and the GPU overlaps them.
    streams = [stream] + [torch.cuda.Stream() for _ in lcs[1:]]
    if args.serial:
        streams = [stream] * len(lcs)

    def step():
        for lc, st in zip(lcs, streams):
            b.gspc_set_stream(st)
            b.gspc_run_layer_chain(lc)
        b.gspc_set_stream(stream)

    # Depth fusion shortens a chain that runs alone (see per_g below), but its
    # kernels hold a whole CU's LDS; with five chains in flight the separate
    # small kernels fill each other's gaps and the step is faster without it.
    b.gspc_set_chain_fusion(1 if args.fusion else 0)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = t1 - t0
    ms_per_step = sec / args.steps * 1e3
    value = macs_step * args.steps / sec / 1e9

    # ---- per-g latency (outside the timed region), library defaults ---------
    b.gspc_set_chain_fusion(1)
    per_g = {}
    for g, ch, lc in zip(GROUPS, chains, lcs):
        reps = max(5, min(50, args.steps))
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for _ in range(reps):
            b.gspc_run_layer_chain(lc)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - ta) / reps * 1e3
        per_g[str(g)] = {"ms": round(ms, 4), "gmacs": round(ch.macs() / ms / 1e6, 1)}

    # ---- roofline of the dominant kernel ------------------------------------
    roofline, roofline_direct = None, None
    kernels = {}
    if not args.no_roofline:
        b.gspc_set_chain_fusion(0)   # this leg times single layers
        reps = 20
        for ch, (packed, bufs) in zip(chains, keep):
            seen = {}
            for l in ch.layers:
                if l.op != "conv":
                    continue
                key = (l.Cin, l.H, l.W, l.Cout, l.KH, l.stride, l.groups, l.src2 >= 0, l.relu)
                if key in seen:
                    seen[key][1] += 1
                    continue
                seen[key] = [l, 1]
            for l, count in seen.values():
                # the same layer `inner` times in one recorded chain: back-to-back
                # launches with no host in the loop
                inner = 10
                one = b.LayerChain([l] * inner, packed, bufs)
                b.gspc_run_layer_chain(one)
                name = b.gspc_last_kernel()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(reps):
                    b.gspc_run_layer_chain(one)
                e1.record()
                torch.cuda.synchronize()
                dur = e0.elapsed_time(e1) / (reps * inner) * 1e-3
                flops, nbytes = layer_flops_bytes(l)
                k = kernels.setdefault(name, {"time": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0,
                                              "compute_bound": False})
                k["time"] += dur * count
                k["flops"] += flops * count
                k["bytes"] += nbytes * count
                k["launches"] += count
                # fp32 ridge of this GPU: 157.3 TFLOP/s / 8 TB/s = 19.7 flop/B
                if flops / nbytes > PEAK_F32_MFMA_TFLOPS * 1e3 / PEAK_HBM_GBS:
                    k["compute_bound"] = True
        name, k = max(kernels.items(), key=lambda kv: kv[1]["time"])
        roofline = _roofline_object(name, k, kernels)
        all_flops = sum(v["flops"] for v in kernels.values())
        roofline["winograd_share_of_macs"] = round(sum(v["flops"] for n, v in kernels.items() if "wino" in n) / all_flops, 4)
        if "wino" in name:
            # the kernel instance with the largest share of the step is the Winograd one: the direct-sum
            # instance with the largest share is reported next to it
            direct = {n: v for n, v in kernels.items() if "wino" not in n}
            if direct:
                dn, dk = max(direct.items(), key=lambda kv: kv[1]["time"])
                roofline_direct = _roofline_object(dn, dk, kernels)

    # ---- HBM side: depthwise 3x3 layers at batch 256, rotating buffers ------------
    roofline_hbm, latency = None, None
    if not args.no_extra:
        from paper_2006_09791_amd import layer_timing
        b.gspc_set_stream(stream)
        shapes = [dw for dw, _ in wl.depthwise_pairs(256)]
        rows = layer_timing.time_layers(shapes, "f32", inner=8, reps=3, rotate=4)
        fam = {}
        for sh, r in zip(shapes, rows):
            f = fam.setdefault(r["kernel"], {"time": 0.0, "bytes": 0.0, "launches": 0})
            f["time"] += r["us"] * 1e-6
            f["bytes"] += layer_timing.layer_bytes(sh, 4)
            f["launches"] += 1
        name, f = max(fam.items(), key=lambda kv: kv[1]["time"])
        ach = f["bytes"] / f["time"] / 1e9
        roofline_hbm = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None, "kernel": name,
                        "workload": "MobileNet-shaped depthwise 3x3 layers (C, HxW) in {(32,112),(64,112),(128,56),(256,28),"
                                    "(512,14),(1024,7)} x stride {1,2}, fp32, N=256, four rotating buffer sets",
                        "layers_served": f["launches"], "avg_launch_us": round(f["time"] / f["launches"] * 1e6, 2),
                        "all_layers_frac": round(sum(v["bytes"] for v in fam.values()) / sum(v["time"] for v in fam.values())
                                                 / 1e9 / PEAK_HBM_GBS, 4)}

        # ---- batch-1 network latency, recorded chains (Tables II-III quantity) ------
        b.gspc_set_chain_fusion(1)
        latency = {}
        nets = [("wrn40x2_style", wl.wrn_chain, GROUPS, 2), ("resnet34_shaped", wl.resnet34_chain, (2, 4, 8, 16, 32), 3)]
        for tag, make, gs, cfg in nets:
            latency[tag] = {}
            for g in gs:
                ch = make(1, g)
                weights = ch.make_weights(cfg)
                packed = [b.gspc_pack_weights(torch.from_numpy(w).to(dev), gg) for w, gg in zip(weights, ch.weight_groups)]
                bufs = [torch.empty(max(n, 1), dtype=torch.float32, device=dev) for n in ch.buf_elems]
                bufs[0].copy_(torch.from_numpy(wl.make_input(ch.input_shape, 1)).reshape(-1))
                lc = b.LayerChain(ch.layers, packed, bufs)
                for _ in range(5):
                    b.gspc_run_layer_chain(lc)
                torch.cuda.synchronize()
                reps = 50
                ta = time.perf_counter()
                for _ in range(reps):
                    b.gspc_run_layer_chain(lc)
                torch.cuda.synchronize()
                latency[tag][str(g)] = round((time.perf_counter() - ta) / reps * 1e3, 4)
                del lc, bufs, packed

    # ---- CPU oracle on a bounded sample -------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
        cores = max(1, min(cores, oracle.max_threads(), 16))


        def time_oracle(n_s, threads, runner):
            total, t_cpu = 0, 0.0
            for g in GROUPS:
                ch = wl.wrn_chain(n_s, g)
                weights = ch.make_weights(2)
                x0 = wl.make_input(ch.input_shape, wl.make_seed(2, 999, g))
                prep = runner(ch, weights, None, threads, prepare=True)
                ta = time.perf_counter()
                runner(ch, weights, x0, threads, prep=prep)
                t_cpu += time.perf_counter() - ta
                total += ch.macs()
            return total, t_cpu

        def run_definition(ch, weights, x0, threads, prepare=False, prep=None):
            if prepare:
                return None
            oracle.run_chain(ch.layers, len(ch.buf_elems), x0, weights, threads=threads)

        def tiles(l):
            cpg, kpg = l.Cin // l.groups, l.Cout // l.groups
            return (max(t for t in (1, 2, 3, 4) if cpg % t == 0), max(t for t in (1, 2, 4, 8, 16) if kpg % t == 0))

        def run_alg1(ch, weights, x0, threads, prepare=False, prep=None):
            # Algorithm 1 with the kernel reshape done ahead of time (Section III-B) and the
            # convolution stage in its vectorised, multi-core schedule; a conv step's residual
            # and ReLU as in oracle.run_chain
            if prepare:
                return [oracle.alg1_pack_kernels(weights[l.wid], l.groups, *tiles(l)) for l in ch.layers if l.op == "conv"]
            bufs = [None] * len(ch.buf_elems)
            bufs[0] = x0
            k = 0
            for l in ch.layers:
                ti, to = tiles(l)
                y = oracle.gspc_alg1(bufs[l.src], weights[l.wid], l.stride, l.pad, l.groups, ti, to, vectorised=True,
                                     threads=threads, packed_w=prep[k])
                k += 1
                if l.src2 >= 0:
                    y = oracle.add(y, bufs[l.src2])
                bufs[l.dst] = oracle.relu(y) if l.relu else y

        total, t_cpu = time_oracle(BATCH, cores, run_definition)
        cpu = {"value": round(total / t_cpu / 1e9, 3), "unit": "GMAC/s", "cores": cores,
               "kind": "oracle",
               "sample": f"same WRN-40-2-style stacks, g in {list(GROUPS)}, batch {BATCH} "
                         f"({total / 1e9:.2f} GMAC, {t_cpu:.1f} s wall)"}
        total1, t1c = time_oracle(1, 1, run_definition)
        cpu["single_thread"] = {"value": round(total1 / t1c / 1e9, 3), "unit": "GMAC/s", "cores": 1, "kind": "oracle",
                                "sample": f"the same stacks at batch 1 ({total1 / 1e9:.2f} GMAC, {t1c:.1f} s wall)"}
        totala, ta_ = time_oracle(BATCH, cores, run_alg1)
        cpu["gspc_alg1_vectorised"] = {
            "value": round(totala / ta_ / 1e9, 3), "unit": "GMAC/s", "cores": cores, "kind": "oracle (timed baseline only)",
            "sample": f"the same stacks at batch {BATCH} through Algorithm 1: kernels packed ahead of time, input and output "
                      f"reshapes timed, T_O <= 16 filters as one fp64 vector, (group, image) pairs over the cores "
                      f"({totala / 1e9:.2f} GMAC, {ta_:.1f} s wall)"}
        totalb, tb_ = time_oracle(1, 1, run_alg1)
        cpu["gspc_alg1_vectorised"]["single_thread"] = round(totalb / tb_ / 1e9, 3)

    out = {
        "metric": "grouped conv2d GMAC/s (Eq. 2 MACs / time), WRN-40-2-style stack swept over g",
        "value": round(value, 1), "unit": "GMAC/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "WRN-40-2-style CIFAR stack, 3x32x32 input, every 3x3 conv grouped, "
                               "fp32, N=64, one pass per g in {1,2,4,8,16} per step",
                   "batch": BATCH, "groups": list(GROUPS), "gmac_per_step": round(macs_step / 1e9, 3),
                   "streams": 1 if args.serial else len(GROUPS), "chain_fusion_in_step": bool(args.fusion)},
        "per_g": per_g,
        "per_g_monotone": all(per_g[str(a)]["ms"] >= per_g[str(c)]["ms"] * 0.97 for a, c in zip(GROUPS, GROUPS[1:])),
        "roofline": roofline,
        "roofline_direct": roofline_direct,
        "roofline_hbm": roofline_hbm,
        "latency_ms": latency,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
