"""Test oracle (never imported by the product): the fill-job Scheduler of Sec. 4.4 and the
event-driven simulation of Sec. 5.1, in plain Python integers.

A job's processing time on a device follows from the device's bubble cycle, the job's profile
and Algorithm 1 (Sec. 4.4: the Scheduler can work out exactly how long any fill job takes on any device).
When a device is free and jobs wait, the job with the largest policy score is submitted to it:
  FIFO      score = -arrival
  SJF       score = 1 / min(j.proc_times)                      (Sec. 4.4, first formula)
  MAKESPAN  score = 1 / max(j.proc_times[i], max(s.rem_times)) (Sec. 4.4, second formula)
Scores are compared exactly (as fractions); ties go to the earlier arrival, then the lower index.
Events are job arrivals and job completions (Sec. 5.1); at an event every idle device is offered
the queue, in device order.
"""
from fractions import Fraction

from oracle import planner as op

FIFO, SJF, MAKESPAN = 0, 1, 2


def job_time(bubbles, F, samples_per_replica, total_samples, iter_ns, fill_ppm=1_000_000, switch_ns=0):
    """Bubble cycles of whole plan passes needed for total_samples, times the main job's iteration
    time: one pass of the plan completes replicas * samples_per_replica samples in
    ceil(len(P) / len(B)) cycles."""
    chunks, k = op.partition_fill_job(bubbles, F, fill_ppm, 0, switch_ns)
    n_fill = sum(1 for b in bubbles if b["fillable"])
    cycles = op.plan_cycles(chunks, n_fill)
    per_pass = k * samples_per_replica
    passes = -(-total_samples // per_pass)
    return passes * cycles * iter_ns


def score(policy, j, jobs, proc, rem, dev):
    if policy == FIFO:
        return Fraction(-jobs[j]["arrival"])
    if policy == SJF:
        return Fraction(1, min(proc[j]))
    if policy == MAKESPAN:
        return Fraction(1, max(proc[j][dev], max(rem)))
    raise ValueError("unknown policy")


def simulate(policy, jobs, proc, n_dev):
    """jobs: list of dicts (arrival); proc[j][i] > 0: processing time of job j on device i.
    Returns (assignment list of (device, start, finish) per job, makespan, sum of completion times
    measured from each job's arrival)."""
    n = len(jobs)
    free_at = [0] * n_dev
    out = [None] * n
    waiting = []
    arrivals = sorted(range(n), key=lambda j: (jobs[j]["arrival"], j))
    nxt = 0
    t = 0
    done = 0
    while done < n:
        # next event: an arrival or the completion of a running job
        cand = []
        if nxt < n:
            cand.append(jobs[arrivals[nxt]]["arrival"])
        cand += [f for f in free_at if f > t]
        if not waiting or all(f > t for f in free_at):
            t = max(t, min(cand)) if cand else t
        while nxt < n and jobs[arrivals[nxt]]["arrival"] <= t:
            waiting.append(arrivals[nxt])
            nxt += 1
        for dev in range(n_dev):
            if free_at[dev] > t or not waiting:
                continue
            rem = [max(f - t, 0) for f in free_at]
            best = max(waiting, key=lambda j: (score(policy, j, jobs, proc, rem, dev), -jobs[j]["arrival"], -j))
            waiting.remove(best)
            out[best] = (dev, t, t + proc[best][dev])
            free_at[dev] = t + proc[best][dev]
            done += 1
    makespan = max(f for _, _, f in out)
    jct = sum(f - jobs[j]["arrival"] for j, (_, _, f) in enumerate(out))
    return out, makespan, jct
