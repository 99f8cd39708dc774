"""Per-layer timing of gspc_conv2d_grouped-shaped work on the current stream.

Each layer is replayed back to back inside one recorded layer chain (no host in
the loop) and timed with events on the launch stream.  Returns rows with the
Eq. 2 MAC count, the algorithmic bytes and the fractions of the nominal MI355X
ceilings (fp32 MFMA 157.3 TFLOP/s, bf16 MFMA 2500 TFLOP/s, HBM 8 TB/s).  Rows of the
Winograd kernel report the executed multiplications (16/36 of Eq. 2's) against the peak.
"""
import numpy as np

from . import binding as b
from . import workloads as wl

PEAK_HBM_GBS = 8000.0
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


def layer_bytes(s, in_bytes):
    ho, wo = wl.out_size(s.H, s.KH, s.stride, s.pad), wl.out_size(s.W, s.KW, s.stride, s.pad)
    return (s.N * s.Cin * s.H * s.W * in_bytes + s.Cout * (s.Cin // s.groups) * s.KH * s.KW * 4
            + s.N * s.Cout * ho * wo * 4)


def time_layers(shapes, dtype="f32", inner=10, reps=10, rotate=1):
    """shapes: list of workloads.ConvShape.  rotate > 1 cycles through that
    many independent input/output buffer sets so that consecutive launches do
    not find their data in cache (for HBM-bandwidth claims)."""
    import torch
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    b.gspc_set_chain_fusion(0)   # the chains below repeat one layer: time it as a single kernel
    rows = []
    for s in shapes:
        ho, wo = b.gspc_output_dims(s.H, s.W, s.KH, s.KW, s.stride, s.pad)
        w = torch.randn((s.Cout, s.Cin // s.groups, s.KH, s.KW), device=dev) * 0.1
        pw = b.gspc_pack_weights(w, s.groups, b.GSPC_BF16 if dtype == "bf16" else b.GSPC_F32)
        n_in, n_out = s.N * s.Cin * s.H * s.W, s.N * s.Cout * ho * wo
        bufs = []
        for _ in range(rotate):
            x = torch.rand(n_in, device=dev) * 2 - 1
            if dtype == "bf16":
                x = b.gspc_pack_input_bf16(x).view(torch.int16)
            bufs += [x, torch.empty(n_out, dtype=torch.float32, device=dev)]
        layers = []
        for i in range(inner):
            r = i % rotate
            layers.append(wl.Layer("conv", 2 * r, -1, 2 * r + 1, s.N, s.Cin, s.H, s.W, s.Cout, s.KH,
                                   s.KW, s.stride, s.pad, s.groups, False, 0))
        lc = b.LayerChain(layers, [pw], bufs)
        b.gspc_run_layer_chain(lc)
        name = b.gspc_last_kernel()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            b.gspc_run_layer_chain(lc)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / (reps * inner) * 1e3
        macs = wl.conv_macs(s)
        nbytes = layer_bytes(s, 2 if dtype == "bf16" else 4)
        row = {
            "layer": f"{s.Cin}->{s.Cout} {s.H}x{s.W} k{s.KH} s{s.stride} g{s.groups} N{s.N}",
            "kernel": name, "us": round(us, 2), "gmacs": round(macs / us / 1e3, 1),
            "tflops": round(2 * macs / us / 1e6, 2), "gbs": round(nbytes / us / 1e3, 1),
            "frac_mfma": round(2 * macs / us / 1e6 / PEAK_TFLOPS[dtype], 4),
            "frac_hbm": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4),
        }
        if name.startswith("conv_wino"):
            # Winograd F(2x2, 3x3) executes 16/36 of the multiplications Eq. 2 counts: `tflops` is an
            # effective rate (no fraction of a peak belongs to it), `frac_mfma` the executed work's share
            row["algorithm"] = "winograd"
            row["frac_mfma"] = round(row["frac_mfma"] * 16.0 / 36.0, 4)
        rows.append(row)
        del bufs, lc
    b.gspc_set_chain_fusion(1)
    return rows


def time_blocks(pairs, inner=8, reps=5, rotate=4):
    """pairs: (depthwise 3x3, pointwise 1x1) workloads.ConvShape pairs, the block of
    the networks of Section IV-A.  Each block is timed twice inside recorded chains,
    as two kernels and with chain fusion (one kernel where the pair qualifies).
    The input and output buffers rotate; the depthwise result has one buffer, which the
    next block overwrites (as in a network that reuses its activation buffers), so a
    fused block need not store it.  Bytes are the block's algorithmic ones:
    input + both weight tensors + pointwise output."""
    import torch
    dev = torch.device("cuda:0")
    b.gspc_set_stream()
    rows = []
    for dw, pw in pairs:
        ho, wo = b.gspc_output_dims(dw.H, dw.W, 3, 3, dw.stride, dw.pad)
        w1 = torch.randn((dw.Cout, 1, 3, 3), device=dev) * 0.3
        w2 = torch.randn((pw.Cout, pw.Cin, 1, 1), device=dev) * 0.1
        packed = [b.gspc_pack_weights(w1, dw.groups), b.gspc_pack_weights(w2, 1)]
        n_in, n_mid, n_out = dw.N * dw.Cin * dw.H * dw.W, dw.N * dw.Cout * ho * wo, pw.N * pw.Cout * ho * wo
        bufs = [torch.empty(n_mid, dtype=torch.float32, device=dev)]
        for _ in range(rotate):
            bufs += [torch.rand(n_in, device=dev) * 2 - 1, torch.empty(n_out, dtype=torch.float32, device=dev)]
        layers = []
        for i in range(inner):
            r = i % rotate
            layers.append(wl.Layer("conv", 1 + 2 * r, -1, 0, dw.N, dw.Cin, dw.H, dw.W, dw.Cout, 3, 3,
                                   dw.stride, dw.pad, dw.groups, True, 0))
            layers.append(wl.Layer("conv", 0, -1, 2 + 2 * r, pw.N, pw.Cin, ho, wo, pw.Cout, 1, 1, 1, 0, 1, True, 1))
        lc = b.LayerChain(layers, packed, bufs)
        row = {"block": f"dw {dw.Cin}@{dw.H}x{dw.W} s{dw.stride} + pw {pw.Cin}->{pw.Cout} N{dw.N}"}
        macs = wl.conv_macs(dw) + wl.conv_macs(pw)
        nbytes = (n_in + n_out + dw.Cout * 9 + pw.Cout * pw.Cin) * 4
        for mode in ("two_kernels", "fused"):
            b.gspc_set_chain_fusion(1 if mode == "fused" else 0)
            b.gspc_run_layer_chain(lc)
            name = b.gspc_last_kernel()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                b.gspc_run_layer_chain(lc)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / (reps * inner) * 1e3
            row[mode] = {"kernel": name, "us": round(us, 2), "tflops": round(2 * macs / us / 1e6, 2),
                         "gbs": round(nbytes / us / 1e3, 1)}
        b.gspc_set_chain_fusion(1)
        rows.append(row)
        del bufs, lc
    return rows
