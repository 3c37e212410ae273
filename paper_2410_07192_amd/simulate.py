"""Scheduler study on synthetic arrivals: the three policies of Sec. 4.4 in the event-driven simulation of
Sec. 5.1 (the one-node analogue of the policy comparison of Sec. 6.2).

    python -m paper_2410_07192_amd.simulate [--jobs 300] [--load 0.8] [--seed 0] > policies.jsonl

One Executor per pipeline stage of one main-job replica (p devices, each with its own bubble cycle).  A job's
processing time on every device comes from the planner (pf_job_time: Algorithm 1 on that device's windows);
pf_sched_simulate then plays the arrivals against each policy.  One JSON line per policy.  Runs on the CPU.

The job trace of the paper is not available: jobs are drawn from three synthetic kinds whose per-node times
are the ones measured on MI355X for the benchmark workloads (encoder inference 0.35 ms per layer, a larger
encoder 1.1 ms per layer, decoder training 0.31 / 1.32 ms per layer forward / backward), with log-normal sizes
and Poisson arrivals scaled to a target load."""
from __future__ import annotations

import argparse
import json
import math
import random

from . import binding as pf

MS = 1_000_000
GIB = 1 << 30


def chain(kind):
    """(nodes as (dur_ns, mem_bytes), samples per replica) of a job kind."""
    if kind == "enc-base-infer":
        return [(int(0.02 * MS), 1 * GIB)] + [(int(0.35 * MS), 2 * GIB)] * 12 + [(int(0.02 * MS), 1 * GIB)], 32
    if kind == "enc-large-infer":
        return [(int(0.03 * MS), 2 * GIB)] + [(int(1.1 * MS), 6 * GIB)] * 24 + [(int(0.03 * MS), 2 * GIB)], 32
    if kind == "dec-small-train":
        return ([(int(0.03 * MS), 6 * GIB)] + [(int(0.31 * MS), 6 * GIB)] * 12 + [(int(0.02 * MS), 6 * GIB)] +
                [(int(3.6 * MS), 6 * GIB)] + [(int(1.32 * MS), 6 * GIB)] * 12 + [(int(0.4 * MS), 6 * GIB)] +
                [(int(0.42 * MS), 6 * GIB)]), 8
    raise ValueError(kind)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stages", type=int, default=16)
    ap.add_argument("--microbatches", type=int, default=32)
    ap.add_argument("--tf-ms", type=float, default=15.0)
    ap.add_argument("--tb-ms", type=float, default=30.0)
    ap.add_argument("--free-gib", type=float, default=16.0)
    ap.add_argument("--jobs", type=int, default=300)
    ap.add_argument("--load", type=float, default=0.8, help="offered work / capacity of the p Executors")
    ap.add_argument("--fill-ppm", type=int, default=900_000)
    ap.add_argument("--switch-ns", type=int, default=100_000)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()

    p, m = args.stages, args.microbatches
    tf, tb = int(args.tf_ms * MS), int(args.tb_ms * MS)
    iter_ns = (m + p - 1) * (tf + tb)
    windows = [pf.pf_schedule_1f1b(p, m, s, tf, tb, int(args.free_gib * GIB), True, 0) for s in range(p)]

    rng = random.Random(args.seed)
    kinds = ["enc-base-infer", "enc-large-infer", "dec-small-train"]
    drawn = []
    for _ in range(args.jobs):
        kind = rng.choices(kinds, weights=[5, 3, 2])[0]
        nodes, spr = chain(kind)
        total = max(spr, int(rng.lognormvariate(math.log(200_000), 1.0)))
        F = pf.nodes_to_c(nodes)
        proc = [pf.pf_job_time(windows[s], F, spr, total, iter_ns, args.fill_ppm, args.switch_ns) for s in range(p)]
        drawn.append((kind, total, proc))
    # Poisson arrivals: the mean job keeps its fastest device busy for mean_best; p devices serve p / mean_best jobs
    # per unit time at full load
    mean_best = sum(min(pr) for _, _, pr in drawn) / len(drawn)
    gap = mean_best / (p * args.load)
    t = 0.0
    jobs = []
    for _ in drawn:
        t += rng.expovariate(1.0 / gap)
        jobs.append(dict(arrival=int(t)))

    for name, code in (("fifo", pf.PF_POLICY_FIFO), ("sjf", pf.PF_POLICY_SJF), ("makespan", pf.PF_POLICY_MAKESPAN)):
        runs, makespan, total_jct = pf.pf_sched_simulate(code, jobs, [pr for _, _, pr in drawn], p)
        jct = sorted(f - j["arrival"] for (_, _, f), j in zip(runs, jobs))
        busy = sum(f - s for _, s, f in runs)
        print(json.dumps({
            "policy": name, "jobs": len(jobs), "devices": p, "load": args.load, "seed": args.seed,
            "makespan_s": makespan * 1e-9, "mean_jct_s": total_jct / len(jobs) * 1e-9,
            "median_jct_s": jct[len(jct) // 2] * 1e-9, "p95_jct_s": jct[int(0.95 * (len(jct) - 1))] * 1e-9,
            "executor_utilisation": busy / (p * makespan),
            "mean_best_proc_s": mean_best * 1e-9, "main_iteration_s": iter_ns * 1e-9}), flush=True)


if __name__ == "__main__":
    main()
