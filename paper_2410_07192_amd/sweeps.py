"""One-GPU sweeps over the Executor's knobs, the analogues of the paper's sensitivity studies: main-job
slowdown and fill throughput against the fraction of each bubble the Executor tries to fill (Sec. 6.1,
Fig. 5), fill throughput against the bubble size and against the free memory (Sec. 6.4, Fig. 10), and
the main job's optimizer-state offload (Sec. 4.2) against the time its gradient synchronisation takes.

    python -m paper_2410_07192_amd.sweeps [--which fill,bubble,memory,offload] > sweeps.jsonl

Every point is one run of bench.py (a child process, so each point starts from a fresh context); one JSON
object per point on stdout: the sweep's name, the knob's value and the fields of bench.py's line that the
study plots."""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KEEP = ("value", "unit", "pct_bubble_filled", "overrun_pct_of_offered", "main_slowdown_pct", "fill_tflops_in_bubbles",
        "replicas_done", "chunks_run")


def run_point(name, knob, value, extra):
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--no-cpu-baseline", *extra]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    rec = {"sweep": name, knob: value}
    if out.returncode != 0:
        rec["error"] = out.stderr.strip().splitlines()[-1] if out.stderr.strip() else f"exit {out.returncode}"
    else:
        line = json.loads(out.stdout.strip().splitlines()[-1])
        rec.update({k: line.get(k) for k in KEEP})
        rec["microbatches_per_layer_visit"] = line.get("config", {}).get("microbatches_per_layer_visit")
        rec["chosen"] = line.get("config", {}).get("chosen")
        rec["copy_wait_pct_of_offered"] = line.get("copy_wait_pct_of_offered")
        if "main_offload" in line:
            rec["main_offload"] = line["main_offload"]
    print(json.dumps(rec), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--which", default="fill,bubble,memory,offload")
    ap.add_argument("--caps", default="0.4,0.5,0.75,1,1.5,2,4,8", help="memory sweep: free GiB inside the bubbles")
    args = ap.parse_args()
    which = set(args.which.split(","))
    if "fill" in which:      # real main-stage kernels (cfg5) with the streamed fill job inside its bubbles
        for ppm in (300_000, 500_000, 680_000, 800_000, 900_000, 980_000):
            run_point("fill_fraction", "fill_ppm", ppm, ["--workload", "cfg5", "--fill-ppm", str(ppm), "--steps", "4",
                                                          "--warmup", "1"])
    if "bubble" in which:    # streamed fill job (cfg3) in explicit bubbles of growing size
        for ms in (5, 10, 20, 40, 80, 160):   # at least 20 bubbles and 3.2 s of them: a batch spans several small ones
            run_point("bubble_size", "bubble_ms", ms, ["--workload", "cfg3", "--bubble-ms", str(ms), "--steps",
                                                        str(max(20, 3200 // ms))])
    if "memory" in which:    # the same job with less and less free memory; the planner may keep the weights resident,
        # or stream them through 3 or 2 slots, with 16, 4 or 1 sequences per microbatch and 1 or 4 microbatches per layer
        # visit (Sec. 4.3: batch size x technique)
        for gib in (float(c) for c in args.caps.split(",")):
            run_point("free_memory", "cap_gib", gib, ["--workload", "cfg3", "--candidates", "all", "--cap-gib", str(gib),
                                                       "--steps", "50"])
    if "offload" in which:   # cfg5 with 1 GiB free: the fill job only fits the windows that the offload enlarges
        for ms in (10, 25, 50, 100, 200, 400):
            run_point("main_offload", "sync_ms", ms, ["--workload", "cfg5", "--main-offload", "--cap-gib", "1", "--sync-ms",
                                                       str(ms), "--steps", "4", "--warmup", "1"])


if __name__ == "__main__":
    main()
