"""Pins of the Scheduler / event-driven simulation checker (oracle/scheduler.py): closed forms, brute force,
invariants and hand-worked examples (Sec. 4.4, Sec. 5.1)."""
import itertools
import random

from oracle import planner as op
from oracle import scheduler as sc


def test_job_time_from_the_plan():
    # one bubble of 100, chain of one node of 10: 9 replicas per pass (9*10 < 100), one cycle per pass
    B = [dict(dur=100, free=5, fillable=1)]
    assert sc.job_time(B, [(10, 5)], samples_per_replica=4, total_samples=36, iter_ns=1000) == 1000
    assert sc.job_time(B, [(10, 5)], 4, 37, 1000) == 2000            # one more sample needs a second pass
    # bubbles 10 and 6, chain of four nodes of 2: 1 replica in 1 cycle (hand example of the planner pins)
    B = [dict(dur=10, free=9, fillable=1), dict(dur=6, free=9, fillable=1)]
    assert sc.job_time(B, [(2, 1)] * 4, 8, 80, 500) == 10 * 500
    # a plan that spills into a second cycle counts two cycles per pass
    B = [dict(dur=8, free=9, fillable=1)]
    chunks, k = op.partition_fill_job(B, [(4, 1), (4, 1)])
    assert (k, len(chunks)) == (1, 2)                                 # 4 < 8 fits, 4 + 4 < 8 does not: second visit
    assert sc.job_time(B, [(4, 1), (4, 1)], 1, 3, 100) == 3 * 2 * 100


def test_sjf_minimises_mean_completion_time_on_one_device():
    rnd = random.Random(1)
    for _ in range(200):
        n = rnd.randint(1, 6)
        jobs = [dict(arrival=0) for _ in range(n)]
        proc = [[rnd.randint(1, 20)] for _ in range(n)]
        out, makespan, jct = sc.simulate(sc.SJF, jobs, proc, 1)
        best = min(sum(itertools.accumulate(proc[j][0] for j in perm)) for perm in itertools.permutations(range(n)))
        assert jct == best and makespan == sum(p[0] for p in proc)


def test_simulation_invariants():
    rnd = random.Random(2)
    for trial in range(300):
        n, d = rnd.randint(1, 8), rnd.randint(1, 3)
        jobs = [dict(arrival=rnd.randint(0, 30)) for _ in range(n)]
        proc = [[rnd.randint(1, 20) for _ in range(d)] for _ in range(n)]
        for policy in (sc.FIFO, sc.SJF, sc.MAKESPAN):
            out, makespan, jct = sc.simulate(policy, jobs, proc, d)
            assert makespan == max(f for _, _, f in out)
            assert jct == sum(f - jobs[j]["arrival"] for j, (_, _, f) in enumerate(out))
            for j, (dev, s, f) in enumerate(out):
                assert s >= jobs[j]["arrival"] and f == s + proc[j][dev]
            for dev in range(d):
                iv = sorted((s, f) for (dv, s, f) in out if dv == dev)
                assert all(b <= c for (_, b), (c, _) in zip(iv, iv[1:]))
            # work conservation: while a job waits, every device is busy
            for j, (dev, s, f) in enumerate(out):
                for dv in range(d):
                    busy = [(a, b) for (x, a, b) in out if x == dv]
                    for pt in [jobs[j]["arrival"]] + [b for a, b in busy if jobs[j]["arrival"] <= b < s]:
                        if pt < s:
                            assert any(a <= pt < b for a, b in busy), (trial, policy, j, dv)
            if policy == sc.FIFO and d == 1:
                order = sorted(range(n), key=lambda j: out[j][1])
                assert order == sorted(range(n), key=lambda j: (jobs[j]["arrival"], j))


def test_hand_examples():
    # two devices, three jobs at time 0.  proc[j] = times on device 0 and 1.
    jobs = [dict(arrival=0)] * 3
    proc = [[10, 4], [6, 6], [3, 9]]
    # SJF ranks by min over devices: job 2 (3), job 0 (4), job 1 (6).  Device 0 takes job 2 (0-3), device 1 takes job 0
    # (0-4); device 0 is free first and takes job 1 (3-9).
    out, makespan, jct = sc.simulate(sc.SJF, jobs, proc, 2)
    assert out == [(1, 0, 4), (0, 3, 9), (0, 0, 3)] and makespan == 9 and jct == 16
    # FIFO: job 0 on device 0 (0-10), job 1 on device 1 (0-6), job 2 on device 1 (6-15)
    out, makespan, _ = sc.simulate(sc.FIFO, jobs, proc, 2)
    assert out == [(0, 0, 10), (1, 0, 6), (1, 6, 15)] and makespan == 15
    # MAKESPAN on device 0 at t=0: rem = [0, 0], scores 1/10, 1/6, 1/3 -> job 2 (0-3); device 1: rem = [3, 0]:
    # max(4,3)=4, max(6,3)=6 -> job 0 (0-4); at t=3 device 0: rem = [0, 1]: job 1, max(6,1)=6 -> (3-9)
    out, makespan, _ = sc.simulate(sc.MAKESPAN, jobs, proc, 2)
    assert out == [(1, 0, 4), (0, 3, 9), (0, 0, 3)] and makespan == 9
    # a late arrival waits for its arrival even if devices idle; ties go to the earlier arrival, then the lower index
    jobs = [dict(arrival=5), dict(arrival=0), dict(arrival=0)]
    out, _, _ = sc.simulate(sc.SJF, jobs, [[2], [7], [7]], 1)
    assert out == [(0, 7, 9), (0, 0, 7), (0, 9, 16)]
