"""Offline tile-table autotuner for libgspc (the search the paper delegates to an
auto-tuner, Section III-C: tile sizes and unrolling per workload, stored ahead of time).

For every layer shape of a workload it times each kernel family / tile configuration the
library can be told to use and writes the winners to a text table; a process that sets
GSPC_TUNE_FILE to that table before loading the library gets those choices instead of
the planners' heuristics.

    python -m paper_2006_09791_amd.autotune --workload wrn --batch 64 --out wrn64.tune

The forcing itself goes through the same table mechanism: a candidate (family, index) is
tried by writing a temporary table that names it for every shape and timing all shapes in
a child process (the library reads the table once per process).  Shapes for which the
planner cannot realise the candidate fall back to the heuristic choice and are recognised
by the kernel name they report.
"""
import argparse
import json
import os
import subprocess
import sys
import tempfile

from . import workloads as wl

# family letter -> (kernel-name prefix, candidate indices)
FAMILIES = {
    "w": ("conv_mfma16w<", range(5)),
    "m": ("conv_mfma16<", range(14)),
    "b": ("conv_mfma16b<", range(7)),
    "q": ("conv_mfma4r<", (1, 2, 4)),
    "x": ("conv_wino<", range(7)),      # Winograd F(2x2, 3x3): fp32, 3x3, stride 1, pad 1
    "r": ("conv_row16", range(9)),      # bf16 row products: 3x3, stride 1, pad 1, at most 16 channels per group
}


def workload_shapes(name, batch):
    if name == "wrn":
        return [s for g in (1, 2, 4, 8, 16) for s in wl.wrn_grouped_shapes(batch, g)], "f32"
    if name == "resnet34":
        return [s for g in (2, 4, 8, 16, 32) for s in wl.resnet34_grouped_shapes(batch, g)], "f32"
    if name == "mobilenet_pw":
        return [pw for _, pw in wl.depthwise_pairs(batch)], "f32"
    if name == "resnet34_bf16":
        return [s for g in (2, 8, 32) for s in wl.resnet34_grouped_shapes(batch, g)], "bf16"
    raise SystemExit(f"unknown workload {name}")


def table_line(s, dtype, family, index):
    return (f"{s.N} {s.Cin} {s.H} {s.W} {s.Cout} {s.KH} {s.KW} {s.stride} {s.pad} {s.groups} "
            f"{1 if dtype == 'bf16' else 0} {family} {index}")


SAMPLE = 2048   # output elements per layer that travel back to the parent for the agreement check


def output_sample(b, torch, s, dtype, k):
    """One launch of layer k on inputs that are the same in every child process; returns an
    evenly spaced sample of the output and the output's RMS."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234 + k)
    x = torch.rand((s.N, s.Cin, s.H, s.W), device="cuda", generator=gen) * 2 - 1
    w = torch.randn((s.Cout, s.Cin // s.groups, s.KH, s.KW), device="cuda", generator=gen) * 0.1
    pw = b.gspc_pack_weights(w, s.groups, b.GSPC_BF16 if dtype == "bf16" else b.GSPC_F32)
    if dtype == "bf16":
        x = b.gspc_pack_input_bf16(x)
    y = b.gspc_conv2d_grouped(x, pw, s.N, s.Cin, s.H, s.W, s.Cout, s.KH, s.KW, s.stride, s.pad, s.groups).flatten()
    torch.cuda.synchronize()
    step = max(1, y.numel() // SAMPLE)
    return y[::step][:SAMPLE].double().cpu().tolist(), float(y.double().pow(2).mean().sqrt())


def probe(workload, batch, inner, reps):
    """Child process: time every shape with whatever table the environment names, and sample
    every shape's output."""
    import torch
    from . import binding as b, layer_timing
    b.load()
    torch.cuda.set_stream(torch.cuda.Stream())
    shapes, dtype = workload_shapes(workload, batch)
    rows = layer_timing.time_layers(shapes, dtype, inner=inner, reps=reps)
    b.gspc_set_stream()
    out = []
    for k, (s, r) in enumerate(zip(shapes, rows)):
        sample, rms = output_sample(b, torch, s, dtype, k)
        out.append({"kernel": r["kernel"], "us": r["us"], "sample": sample, "rms": rms})
    print(json.dumps(out))


def agrees(cand, base, tol=1e-5):
    """A candidate's sampled output against the heuristic choice's (GPU against GPU, same inputs):
    max difference relative to the output's RMS.  The kernels differ in summation order only,
    which stays near 1e-6; a table must never select a configuration that computes something else."""
    if len(cand["sample"]) != len(base["sample"]):
        return False
    den = max(base["rms"], 1e-30)
    return max(abs(a - c) for a, c in zip(base["sample"], cand["sample"])) / den <= tol


def run_child(args, table_path):
    env = dict(os.environ)
    env.pop("GSPC_TUNE_FILE", None)
    if table_path:
        env["GSPC_TUNE_FILE"] = table_path
    cmd = [sys.executable, "-m", "paper_2006_09791_amd.autotune", "--probe", "--workload", args.workload,
           "--batch", str(args.batch), "--inner", str(args.inner), "--reps", str(args.reps)]
    out = subprocess.run(cmd, env=env, check=True, capture_output=True, text=True).stdout
    return json.loads(out.strip().splitlines()[-1])


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="wrn", choices=["wrn", "resnet34", "resnet34_bf16", "mobilenet_pw"])
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--inner", type=int, default=10)
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--min-gain", type=float, default=0.03,
                    help="keep an entry only if it beats the heuristic choice by this fraction")
    ap.add_argument("--tol", type=float, default=None,
                    help="largest difference (relative to the output RMS) between a candidate's output and the heuristic "
                         "choice's; default 1e-5 (fp32), 1e-4 (bf16, Winograd candidates)")
    ap.add_argument("--out", default=None, help="table file to write (default: stdout)")
    ap.add_argument("--probe", action="store_true", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.probe:
        probe(args.workload, args.batch, args.inner, args.reps)
        return 0

    shapes, dtype = workload_shapes(args.workload, args.batch)
    base = run_child(args, None)
    best = [{"family": None, "index": None, "us": r["us"], "kernel": r["kernel"]} for r in base]
    rejected = 0
    with tempfile.TemporaryDirectory() as tmp:
        # the bf16 kernel exists for bf16 inputs only, the resident-filter and Winograd kernels for fp32 only
        for fam in (("b", "r", "m", "q") if dtype == "bf16" else ("w", "m", "q", "x")):
            prefix, indices = FAMILIES[fam]
            for idx in indices:
                path = os.path.join(tmp, f"{fam}{idx}.tune")
                with open(path, "w") as f:
                    f.write("\n".join(table_line(s, dtype, fam, idx) for s in shapes) + "\n")
                rows = run_child(args, path)
                for k, r in enumerate(rows):
                    # a candidate counts only where the planner took it: its family's kernel, and
                    # not the instance the heuristics pick anyway (that would be timing noise)
                    if r["kernel"].startswith(prefix) and r["kernel"] != base[k]["kernel"] and r["us"] < best[k]["us"]:
                        tol = args.tol if args.tol is not None else (1e-4 if dtype == "bf16" or fam == "x" else 1e-5)
                        if not agrees(r, base[k], tol):
                            print(f"# rejected {fam}:{idx} for layer {k}: output differs from the heuristic choice's",
                                  file=sys.stderr, flush=True)
                            rejected += 1
                            continue
                        best[k] = {"family": fam, "index": idx, "us": r["us"], "kernel": r["kernel"]}
                print(f"# tried {fam}:{idx}", file=sys.stderr, flush=True)
    lines = [f"# libgspc tile table, workload {args.workload}, batch {args.batch}, dtype {dtype}",
             "# N Cin H W Cout KH KW stride pad groups dtype family index   (us: heuristic -> tuned)"]
    t0 = t1 = 0.0
    for s, b0, b1 in zip(shapes, base, best):
        t0 += b0["us"]
        if b1["family"] is not None and b1["us"] < b0["us"] * (1.0 - args.min_gain):
            lines.append(f"{table_line(s, dtype, b1['family'], b1['index'])}   # {b0['us']:.2f} -> {b1['us']:.2f}  "
                         f"{b0['kernel']} -> {b1['kernel']}")
            t1 += b1["us"]
        else:
            t1 += b0["us"]
    lines.append(f"# sum over the layers: {t0:.1f} us with the heuristics, {t1:.1f} us with this table; "
                 f"{rejected} candidate measurements rejected because their output differed")
    text = "\n".join(lines) + "\n"
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
