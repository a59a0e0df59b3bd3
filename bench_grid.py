#!/usr/bin/env python3
"""The paper's experiment grid on one MI355X (Section 4.1: bCol = cCol in {32, 64, 128}, single
and double precision, every matrix) over the five synthetic configurations that stand in for its
matrix collection, plus the tile-size sweep that stands in for its step-1 / step-2 ablation.

    python bench_grid.py [--configs 1,2,3,4,5] [--widths 32,64,128] [--dtypes f32,f64]
                         [--sweep-config K --sweep ct_size=64,128,256 | col_slice=16,32,64
                          [--sweep-args "--width 128 --dtype f64"]]
                         [--ablation]
                         [--steps K] [--warmup W] [--out table.md]

--ablation is the paper's ablation (Section 4.2, "Ablation Study": step 1 alone, then with step 2)
per configuration: Algorithm 1 with step 1 only (TF_FLAG_NO_SPLIT) at tile sizes 64 ... 2048 (a
tile that does not fit the fast memory makes the plan fail: "does not fit"), step 1 + step 2 from
the paper's ctSize = 2048, and the library's own choice (no tile parameters).

Every grid point is one run of bench.py in a child process (cache-cold rotation, no CPU leg);
this script only collects the JSON lines and prints a table (markdown) with one JSON line per
point on stderr.
"""
import argparse
import json
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def run_point(extra, steps, warmup):
    cmd = [sys.executable, os.path.join(HERE, "bench.py"), "--no-cpu", "--steps", str(steps),
           "--warmup", str(warmup)] + extra
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        return dict(error=(r.stderr.strip().splitlines() or ["failed"])[-1][:160])
    return json.loads(r.stdout.strip().splitlines()[-1])


def row_of(label, d):
    if "error" in d:
        return f"| {label} | failed: {d['error']} |||||||"
    k = d["kernels_ms"]
    return (f"| {label} | {d['ms_per_step']:.4f} | {d['unfused_ms_per_step']:.4f} | "
            f"{d['speedup_vs_unfused']:.2f} | {d['value']:.0f} | {d['hbm_alg_gbs']:.0f} | "
            f"{k['wavefront0']:.4f} / {k['wavefront1']:.4f} | "
            f"{d['fused_ratio']['rows']:.2f} / {d['fused_ratio']['nnz']:.2f} | "
            f"{d['schedule']['tiles']} x {d['schedule']['col_slice']} |")


HEAD = ("| point | fused ms | unfused ms | speedup | useful GFLOP/s | algorithmic GB/s | "
        "wavefront 0 / 1 ms | fused rows / nnz | tiles x slice |\n|---|---|---|---|---|---|---|---|---|")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--widths", default="32,64,128")
    ap.add_argument("--dtypes", default="f32,f64")
    ap.add_argument("--sweep-config", type=int, default=0)
    ap.add_argument("--sweep", default="", help="name=v1,v2,...  (ct_size, col_slice or p)")
    ap.add_argument("--sweep-args", default="", help="further bench.py arguments of a sweep, "
                                                     "e.g. '--width 128 --dtype f64'")
    ap.add_argument("--ablation", action="store_true")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--out", default="")
    a = ap.parse_args()
    lines = [HEAD]
    if a.ablation:
        for cfg in a.configs.split(","):
            points = [(f"step 1 only, t = {t}", ["--ct-size", str(t), "--p", "1", "--no-split"])
                      for t in (64, 128, 256, 512, 1024, 2048)]
            points.append(("steps 1 + 2, ctSize = 2048", ["--ct-size", "2048", "--p", "1"]))
            points.append(("library default", []))
            for label, extra in points:
                d = run_point(["--config", cfg] + extra, a.steps, a.warmup)
                if "error" in d and "does not fit" in d["error"]:
                    d["error"] = "does not fit the fast memory"
                label = f"cfg{cfg} {label}"
                print(json.dumps(dict(point=label, result=d)), file=sys.stderr, flush=True)
                lines.append(row_of(label, d))
    elif a.sweep_config:
        name, vals = a.sweep.split("=")
        for v in vals.split(","):
            d = run_point(["--config", str(a.sweep_config), "--" + name.replace("_", "-"), v] +
                          a.sweep_args.split(), a.steps, a.warmup)
            print(json.dumps(dict(point=f"cfg{a.sweep_config} {name}={v}", result=d)),
                  file=sys.stderr, flush=True)
            lines.append(row_of(f"cfg{a.sweep_config} {name}={v}", d))
    else:
        for cfg in a.configs.split(","):
            for dt in a.dtypes.split(","):
                for w in a.widths.split(","):
                    d = run_point(["--config", cfg, "--width", w, "--dtype", dt], a.steps,
                                  a.warmup)
                    label = f"cfg{cfg} {dt} {w}"
                    print(json.dumps(dict(point=label, result=d)), file=sys.stderr, flush=True)
                    lines.append(row_of(label, d))
    text = "\n".join(lines)
    print(text, flush=True)
    if a.out:
        with open(a.out, "w") as f:
            f.write(text + "\n")


if __name__ == "__main__":
    main()
