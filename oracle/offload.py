"""CPU checker for the main job's optimizer-state offload plan.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this file; the
product path never does, and it shares no code with the native library.  Integer arithmetic
on Python ints (ns, bytes, bytes per second).

What it follows (Sec. 4.2, "Main job offloading", and the bubble instruction of "Bubble
signaling"): the moment estimates of the main job's optimizer are only needed in the optimizer
update, so they can leave the device while the iteration runs.  The copies to the host run
beside the forward passes, the copies back beside the gradient synchronisation, on a stream of
their own, and a bubble instruction first waits for the copies still under way.  What has left
the device by then is memory the fill job may use in that bubble.

Readings where the paper is silent (each is listed in the design notes):
  - one slice leaves with every forward instruction; a slice is no longer than what the
    device-to-host rate moves in t_f, so the copy is over when its forward pass is and no
    bubble instruction ever waits;
  - everything that left comes back during the gradient synchronisation, which follows the
    stage's last backward pass and lasts sync_ns: the total is no more than the host-to-device
    rate moves in sync_ns, so the optimizer update never waits either;
  - sizes are multiples of `align` bytes (256); what does not fit stays on the device;
  - the forwards are served first to last, each taking a full slice until the total is used up;
  - the fill-drain window comes after the optimizer update (the state is back), so it gains
    nothing; every other window gains the slices of the forwards that precede it in the stage's
    1F1B program.
"""
from __future__ import annotations

from oracle.planner import stage_program_1f1b

NS = 1_000_000_000


def bytes_in(rate_bytes_per_s, dur_ns, align=256):
    """Largest multiple of `align` that `rate` moves in `dur_ns`."""
    return (rate_bytes_per_s * dur_ns // NS) // align * align


def offload_slices(state_bytes, m, tf, sync_ns, d2h_rate, h2d_rate, align=256):
    """Bytes that leave the device with each of the m forward instructions of an iteration."""
    assert state_bytes >= 0 and m >= 1 and tf > 0 and sync_ns >= 0 and d2h_rate >= 0 and h2d_rate >= 0
    per_fwd = bytes_in(d2h_rate, tf, align)
    total = min(state_bytes // align * align, m * per_fwd, bytes_in(h2d_rate, sync_ns, align))
    out = []
    left = total
    for _ in range(m):
        c = min(per_fwd, left)
        out.append(c)
        left -= c
    return out


def extra_free_bytes(p, m, s, slices):
    """Bytes of optimizer state that are off the device in each idle window of stage s (windows in
    the order of windows_1f1b / the BUBBLE instructions of stage_program_1f1b)."""
    assert len(slices) == m
    gone = 0
    out = []
    for op, j in stage_program_1f1b(p, m, s):
        if op == "F":
            gone += slices[j]
        elif op == "BUBBLE":
            out.append(gone)
    if s > 0:
        out[-1] = 0          # fill-drain: after gradient synchronisation and the optimizer update
    return out
