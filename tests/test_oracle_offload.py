"""Pins for the oracle of the main job's optimizer-state offload plan (Sec. 4.2, "Main job offloading"):
a hand example, closed forms per window kind, a copy-engine timetable built from the 1F1B start times
(independent of the oracle's walk over the stage program), and maximality of the offloaded total."""
import random

import pytest

from oracle import offload as O
from oracle import planner as P

NS = 10**9


def ceil_div(a, b):
    return -(-a // b)


def forward_starts(p, m, s, tf, tb):
    """Start time of forward j on stage s in the 1F1B timetable with zero communication."""
    nf0 = min(p - s, m)
    first_b = p * tf + (p - 1 - s) * tb
    t = [(s + j) * tf for j in range(nf0)]
    t += [first_b + i * (tf + tb) + tb for i in range(m - nf0)]
    return t


def test_hand_example():
    # 1 ms forwards; 1 024 000 B/s to the host = 1024 B per forward; 2 560 000 B/s back in a 1 ms
    # synchronisation = 2560 B in all; 10 000 B of state (9984 after alignment); 4 microbatches
    sl = O.offload_slices(10_000, 4, 10**6, 10**6, 1_024_000, 2_560_000)
    assert sl == [1024, 1024, 512, 0]
    # stage 2 of 4: two warm-up forwards before the fwd-bwd window, one gap in the cool-down, fill-drain
    assert O.extra_free_bytes(4, 4, 2, sl) == [2048, 2560, 0]
    # stage 1: three warm-up forwards, two gaps
    assert O.extra_free_bytes(4, 4, 1, sl) == [2560, 2560, 2560, 0]
    # stage 0 has no fill-drain window; the last stage has no fwd-bwd window and no gaps
    assert O.extra_free_bytes(4, 4, 0, sl) == [2560, 2560, 2560, 2560]
    assert O.extra_free_bytes(4, 4, 3, sl) == [0]


def test_limits_one_at_a_time():
    tf = 15 * 10**6
    big = 10**12
    # the state itself is the limit
    sl = O.offload_slices(1000 * 256 + 17, 8, tf, 10**9, big, big)
    assert sum(sl) == 1000 * 256 and sl[0] == 1000 * 256 and sl[1:] == [0] * 7
    # the forwards are the limit: every forward carries a full slice
    per = (50 * 10**9 * tf // NS) // 256 * 256
    sl = O.offload_slices(10**13, 8, tf, 10**9, 50 * 10**9, 10**15)
    assert sl == [per] * 8
    # the synchronisation is the limit
    sl = O.offload_slices(10**13, 8, tf, 10**7, 50 * 10**9, 40 * 10**9)
    assert sum(sl) == (40 * 10**9 * 10**7 // NS) // 256 * 256
    # nothing moves without a rate or without a synchronisation to bring it back in
    assert O.offload_slices(10**9, 4, tf, 10**8, 0, big) == [0] * 4
    assert O.offload_slices(10**9, 4, tf, 0, big, big) == [0] * 4
    assert O.offload_slices(10**9, 4, tf, 10**8, big, 0) == [0] * 4


@pytest.mark.parametrize("seed", range(40))
def test_against_the_timetable(seed):
    rng = random.Random(1000 + seed)
    p = rng.randint(1, 8)
    m = rng.randint(1, 12)
    s = rng.randrange(p)
    tf = rng.randint(1, 40) * 10**5
    tb = rng.randint(1, 80) * 10**5
    sync = rng.choice([0, rng.randint(1, 50) * 10**5])
    d2h = rng.choice([0, rng.randint(1, 64) * 10**8])
    h2d = rng.randint(1, 64) * 10**8
    state = rng.randint(0, 1 << 34)
    align = 256
    sl = O.offload_slices(state, m, tf, sync, d2h, h2d)
    total = sum(sl)
    per = max(sl)
    assert len(sl) == m and all(c % align == 0 and c >= 0 for c in sl)
    # full slices first, then a remainder, then nothing
    nz = [c for c in sl if c]
    assert sl == nz + [0] * (m - len(nz)) and all(c == per for c in nz[:-1])
    # the three bounds hold ...
    assert total <= state
    assert all(c * NS <= d2h * tf for c in sl)            # each copy is over within t_f
    assert total * NS <= h2d * sync                       # the way back fits the synchronisation
    # ... and one more aligned block would break one of them: the largest aligned slice that still
    # copies within t_f is found by search, not by the oracle's formula
    c_max = 0
    step = 1 << 40
    while step >= align:
        if (c_max + step) * NS <= d2h * tf:
            c_max += step
        step >>= 1
    more = total + align
    assert more > state or more * NS > h2d * sync or more > m * c_max
    if len(nz) > 1:
        assert per == c_max

    # copy engine: copy j starts with forward j (or when copy j-1 ends) and is over with its forward
    starts = forward_starts(p, m, s, tf, tb)
    end_prev = 0
    ends = []
    for j in range(m):
        st = max(starts[j], end_prev)
        en = st + (ceil_div(sl[j] * NS, d2h) if sl[j] else 0)
        assert en <= starts[j] + tf
        ends.append(en)
        end_prev = en
    extra = O.extra_free_bytes(p, m, s, sl)
    wins = P.windows_1f1b(p, m, s, tf, tb, 0)
    assert len(extra) == len(wins)
    for k, w in enumerate(wins):
        if w["kind"] == P.KIND_FILL_DRAIN:
            assert extra[k] == 0
            continue
        # everything launched before the window opened has also ended by then: no wait at the bubble instruction
        launched = sum(sl[j] for j in range(m) if starts[j] < w["start"])
        landed = sum(sl[j] for j in range(m) if ends[j] <= w["start"])
        assert launched == landed == extra[k]
        if w["kind"] == P.KIND_FWD_BWD:
            assert extra[k] == min(total, min(p - s, m) * per)
        else:
            assert extra[k] == total      # gaps only occur in the cool-down, after the last forward
