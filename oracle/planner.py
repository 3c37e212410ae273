"""CPU checker for the bubble planner.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain reference the tests compare the native planner
against.  Only tests/, the smoke check and the benchmark's cpu_baseline leg
may import it; the product path never does.  It shares no code with the
native library.  All arithmetic is on Python integers (ns, bytes, ppm), so
"bit-exact" has a plain meaning.

What it follows:
  * bubble windows of a unidirectional synchronous schedule: the idle
    fraction (p-1)/(m+p-1) (Sec. 2.1) and the fwd-bwd / fill-drain bubble
    lengths of the 1F1B and GPipe schedules (Sec. 4.5, "Main job pipeline
    schedule");
  * the partitioning procedure of Algorithm 1 (Sec. 4.3), taken in the
    paper's order: replicate the chain, then pack source nodes greedily
    into bubbles that cycle;
  * the choice of the configuration of maximum throughput (Sec. 4.1
    "Putting together", Sec. 4.3 "Execution plan").

Readings where the paper is silent (each is listed in the design notes):
  - stages are 0-based; communication, gradient-sync and optimizer time are 0;
  - time tests are strict (<), the memory test is <=, exactly as in the
    listing of Algorithm 1; memory is tested per node;
  - the share of each bubble that the Executor is allowed to fill (Sec. 6.1) scales
    every bubble duration by fill_ppm/1e6 with floor division, and a fixed
    per-bubble switch cost may be subtracted;
  - a node that fits no bubble would make Algorithm 1 loop forever; here the
    procedure stops with Infeasible after len(B) consecutive empty partitions
    (a first visit shortened by first_dur is not one of them: it says nothing
    about what a whole bubble holds);
  - only bubbles flagged fillable take part; P[i] runs in the
    ((first + i) mod n)-th fillable bubble of cycle (first + i) div n.
"""
from __future__ import annotations

KIND_FWD_BWD = 0
KIND_GAP = 1
KIND_FILL_DRAIN = 2
KIND_EXPLICIT = 3


class Infeasible(Exception):
    """Some node fits no bubble of the cycle (first such node in .node)."""

    def __init__(self, node):
        super().__init__(f"node {node} fits no bubble")
        self.node = node


def iteration_time(p, m, tf, tb):
    """Length of one main-job iteration with zero communication: (m+p-1)(t_f+t_b);
    the per-stage idle time is the fraction (p-1)/(m+p-1) of it (Sec. 2.1)."""
    return (m + p - 1) * (tf + tb)


def windows_1f1b(p, m, s, tf, tb, free_bytes, fill_gaps=True, min_window=0):
    """Idle windows of stage s in one steady-state cycle of a 1F1B schedule.

    Time origin: the global start of the iteration.  Stage s runs
    min(p-s, m) forwards back to back from s*t_f, then idles until the first
    gradient arrives (the fwd-bwd bubble, Sec. 4.5), alternates backward and
    forward, idles t_f before each cool-down backward (the non-contiguous
    bubbles of Sec. 4.5), and finally idles s*(t_f+t_b) until its first forward
    of the next iteration (the fill-drain bubble).

    Returns a list of dicts (start, dur, free, kind, fillable), in time order,
    zero-length windows dropped.  Contiguous bubbles are always fillable; the
    t_f-long gaps only when fill_gaps is set and they last >= min_window.
    """
    assert p >= 1 and m >= 1 and 0 <= s < p and tf >= 0 and tb >= 0
    T = iteration_time(p, m, tf, tb)
    w = min(p - s - 1, m)
    out = []

    def emit(start, end, kind):
        dur = end - start
        if dur <= 0:
            return
        if kind == KIND_GAP:
            fillable = 1 if (fill_gaps and dur >= min_window) else 0
        else:
            fillable = 1
        out.append(dict(start=start, dur=dur, free=free_bytes, kind=kind, fillable=fillable))

    first_b = p * tf + (p - 1 - s) * tb            # start of backward of microbatch 0
    emit((s + min(p - s, m)) * tf, first_b, KIND_FWD_BWD)
    j0 = (m - w) if w < m else 1
    for j in range(j0, m):                          # idle t_f before backward j
        a = first_b + (j - 1) * (tf + tb) + tb      # end of backward j-1
        emit(a, a + tf, KIND_GAP)
    emit(first_b + (m - 1) * (tf + tb) + tb, T + s * tf, KIND_FILL_DRAIN)
    return out


def windows_gpipe(p, m, s, tf, tb, free_bytes):
    """Idle windows of stage s under GPipe (all forwards, then all backwards):
    fwd-bwd bubble of (p-s-1)(t_f+t_b) and the same fill-drain bubble as 1F1B
    (Sec. 4.5)."""
    assert p >= 1 and m >= 1 and 0 <= s < p
    T = iteration_time(p, m, tf, tb)
    out = []
    fb = (p - s - 1) * (tf + tb)
    if fb > 0:
        out.append(dict(start=(s + m) * tf, dur=fb, free=free_bytes, kind=KIND_FWD_BWD, fillable=1))
    fd = s * (tf + tb)
    if fd > 0:
        out.append(dict(start=T + s * tf - fd, dur=fd, free=free_bytes, kind=KIND_FILL_DRAIN, fillable=1))
    return out


def effective_durations(bubbles, fill_ppm=1_000_000, switch_ns=0):
    """Durations the packing may use: floor(dur*fill_ppm/1e6) - switch_ns, not below 0
    (the fill-fraction knob of Sec. 6.1)."""
    eff = []
    for b in bubbles:
        e = (b["dur"] * fill_ppm) // 1_000_000 - switch_ns
        eff.append(e if e > 0 else 0)
    return eff


def partition_fill_job(bubbles, F, fill_ppm=1_000_000, first_bubble=0, switch_ns=0, first_dur=None):
    """Algorithm 1: partition a fill job onto the bubble cycle.

    first_dur (Sec. 4.3, a job that is handed over when the previous one completes, i.e. in
    the middle of a bubble): the first visit of the first bubble only lasts first_dur; the
    fill fraction and the switch time apply to it like to any bubble.  Later visits and the
    replication count use the bubble's own duration.

    bubbles: list of dicts with dur, free, fillable.   F: list of (dur, mem).
    Returns (chunks, replicas) where each chunk is a dict
    (bubble, cycle, node_begin, node_end, dur, mem); node indices run over the
    replicated chain F' = F * replicas; bubble is the index into `bubbles`.
    """
    idx = [i for i, b in enumerate(bubbles) if b["fillable"]]
    n = len(idx)
    if n == 0 or len(F) == 0:
        raise ValueError("empty bubble cycle or empty chain")
    if not (0 <= first_bubble < n):
        raise ValueError("first_bubble out of range")
    eff_all = effective_durations(bubbles, fill_ppm, switch_ns)
    B = [eff_all[i] for i in idx]
    M = [bubbles[i]["free"] for i in idx]

    # replicate while one more copy still fits below the total bubble time
    dur_F = sum(d for d, _ in F)
    total_B = sum(B)
    replicas = 1
    while replicas * dur_F + dur_F < total_B:
        replicas += 1
    Fp = list(F) * replicas

    chunks = []
    pos = 0
    i = first_bubble
    slot = first_bubble
    empty_run = 0
    while pos < len(Fp):
        begin = pos
        dur = 0
        mem = 0
        limit = B[i]
        if first_dur is not None and not chunks:
            limit = max(first_dur * fill_ppm // 1_000_000 - switch_ns, 0)
        while pos < len(Fp) and dur + Fp[pos][0] < limit and Fp[pos][1] <= M[i]:
            dur += Fp[pos][0]
            mem = max(mem, Fp[pos][1])
            pos += 1
        chunks.append(dict(bubble=idx[i], cycle=slot // n, node_begin=begin, node_end=pos,
                           dur=dur, mem=mem))
        if pos == begin:
            # the shortened first visit says nothing about what a whole bubble holds: only full visits count
            if not (first_dur is not None and len(chunks) == 1):
                empty_run += 1
                if empty_run >= n:
                    raise Infeasible(pos % len(F))
        else:
            empty_run = 0
        i = (i + 1) % n
        slot += 1
    return chunks, replicas


def plan_cycles(chunks, n_fillable):
    """Bubble cycles a plan occupies: ceil(len(P) / len(B))."""
    return -(-len(chunks) // n_fillable)


def choose_configuration(bubbles, configs, fill_ppm=1_000_000, first_bubble=0, switch_ns=0):
    """Plan every configuration and keep the one of maximum throughput
    samples*replicas / cycles.  configs: list of dicts (F, samples).  Ties go to
    the smaller peak memory, then to the lower index.  Infeasible configurations
    are skipped; returns (best_index, plans) with plans[c] = None or
    (chunks, replicas, cycles)."""
    n_fill = sum(1 for b in bubbles if b["fillable"])
    plans = []
    best = -1
    best_key = None
    for c, cfg in enumerate(configs):
        try:
            chunks, k = partition_fill_job(bubbles, cfg["F"], fill_ppm, first_bubble, switch_ns)
        except Infeasible:
            plans.append(None)
            continue
        cyc = plan_cycles(chunks, n_fill)
        plans.append((chunks, k, cyc))
        num = cfg["samples"] * k
        peak = max(ch["mem"] for ch in chunks)
        if best < 0:
            best, best_key = c, (num, cyc, peak)
            continue
        bn, bc, bp = best_key
        lhs, rhs = num * bc, bn * cyc          # num/cyc  vs  bn/bc
        if lhs > rhs or (lhs == rhs and peak < bp):
            best, best_key = c, (num, cyc, peak)
    return best, plans


def choose_configuration_stream(bubbles, configs, horizon_cycles, fill_ppm=1_000_000, first_bubble=0, switch_ns=0):
    """Configuration choice when jobs of one kind follow each other (Sec. 4.3: the Executor takes the
    next fill job when one completes, in the middle of a bubble).  Reading: a plan of one job counts
    the rest of its last bubble as used, so configuration c is judged on a run of
    r_c = max(1, ceil(horizon_cycles * U / dur(F_c))) jobs back to back, U = the summed usable duration
    of one bubble cycle; the run is one long chain (F_c repeated r_c times, samples * r_c) and the runs
    are compared like single jobs in choose_configuration.
    Returns (best_index, runs, plans) with plans as in choose_configuration."""
    U = sum(e for e, b in zip(effective_durations(bubbles, fill_ppm, switch_ns), bubbles) if b["fillable"])
    runs, long_cfgs = [], []
    for cfg in configs:
        dur = sum(n[0] for n in cfg["F"])
        r = max(1, -(-(horizon_cycles * U) // dur)) if dur > 0 else 1
        runs.append(r)
        long_cfgs.append(dict(F=list(cfg["F"]) * r, samples=cfg["samples"] * r))
    best, plans = choose_configuration(bubbles, long_cfgs, fill_ppm, first_bubble, switch_ns)
    return best, runs, plans


# --------------------------------------------------------------------------------------
# chain of graph nodes for a transformer fill job (Sec. 4.3: "linearizes the computational
# graph and its profiles, turning it into a sequence of nodes with sequential dependency")

OP_EMBED, OP_LAYER_FWD, OP_FINAL_LN, OP_HEAD_LOSS, OP_LAYER_BWD, OP_OPT = range(6)


def layer_param_count(d, f):
    """Matrices 4d^2 + 2df, biases 3d+d+f+d, LayerNorm 4d."""
    return 4 * d * d + 2 * d * f + (3 * d + d + f + d) + 4 * d


def chain_nodes(n_layers, vocab, g, training):
    """Node list (op, layer, mb_first, mb_count) of one replica = g microbatches: the job's graph
    flattened into a chain (Sec. 4.3).  Inference: [embedding] + one node per layer + final
    LayerNorm.  Training adds the head with its loss, one recompute-and-backward node per layer
    (last layer first) and the optimizer node.  Durations and memory are profiled inputs of the
    Executor (Sec. 4.3), so they are not part of this list."""
    nodes = []
    if vocab > 0 or training:
        nodes.append((OP_EMBED, -1, 0, g))
    for l in range(n_layers):
        nodes.append((OP_LAYER_FWD, l, 0, g))
    nodes.append((OP_FINAL_LN, -1, 0, g))
    if training:
        nodes.append((OP_HEAD_LOSS, -1, 0, g))
        for l in reversed(range(n_layers)):
            nodes.append((OP_LAYER_BWD, l, 0, g))
        nodes.append((OP_OPT, -1, 0, g))
    return nodes


def footprint_bounds(n_layers, d, n_heads, f, seq, batch, vocab, esize, g, streamed, n_slots, training):
    """(lower, upper) bounds in bytes on the HBM a layer-visit node of the job may report, from
    counts of parameters and activations only (Sec. 4.3: a node's memory requirement is a
    profiled input, tested against the bubble's free memory; Sec. 3.2 item 3: model, optimizer
    state and activations are what occupies it).  No buffer list of any implementation enters.

    lower: what the method itself keeps in HBM -- the parameters that stay on the device (all
    layers, or n_slots layers when streamed; embeddings) in the storage type, the g hidden-state
    tensors carried between bubbles, and for training fp32 master weights, two Adam moments and a
    gradient accumulator per parameter plus one checkpoint per layer input and microbatch.
    upper: lower plus a generous allowance for working memory -- every intermediate tensor of one
    layer visit of one microbatch (LayerNorm output, Q, K, V, attention output, projection output,
    FFN intermediate) once for inference and four times for training (forward, saved for backward,
    gradient, transposed operand), a second storage-type copy of the parameters (transposed
    weights), two logits-sized tensors for the head, and 3 % + 48 MiB of padding and small
    per-token statistics."""
    T = batch * seq
    n_layer = layer_param_count(d, f)
    n_emb = (vocab * d + seq * d if vocab > 0 else 0) + 2 * d
    on_device_layers = n_slots if streamed else n_layers
    act = T * d * esize
    inter = T * (6 * d + f) * esize
    if not training:
        lower = (on_device_layers * n_layer + n_emb) * esize + g * act
        upper = lower + inter
    else:
        n_all = n_layers * n_layer + n_emb
        lower = n_all * (esize + 16) + g * (n_layers + 1) * act
        upper = lower + n_all * esize + 4 * inter + 3 * g * act + 2 * T * (vocab + 64) * esize
    return lower, upper + upper * 3 // 100 + (48 << 20)


# ---------------------------------------------------------------------------------------------
# Bubble characterisation by the doubling probe (Sec. 4.2)
# ---------------------------------------------------------------------------------------------
def stage_program_1f1b(p, m, s):
    """Instruction list of stage s for one iteration, 1F1B order: ("F", j), ("B", j) and
    ("BUBBLE", k) where the stage idles in the steady state (k numbers the idle windows of
    windows_1f1b in time order; the fill-drain bubble, if any, is the last entry)."""
    prog = []
    nf0 = min(p - s, m)
    for j in range(nf0):
        prog.append(("F", j))
    k = 0
    # the fwd-bwd window exists when the first gradient arrives after the last warm-up forward ends
    if p - s - 1 > 0:
        prog.append(("BUBBLE", k))
        k += 1
    fnext = nf0
    fwd_before = True
    for j in range(m):
        if not fwd_before:
            prog.append(("BUBBLE", k))
            k += 1
        prog.append(("B", j))
        fwd_before = False
        if fnext < m:
            prog.append(("F", fnext))
            fnext += 1
            fwd_before = True
    if s > 0:
        prog.append(("BUBBLE", k))
        k += 1
    return prog


def pipeline_period_with_waits(p, m, tf, tb, s, waits, iterations=4):
    """Steady-state iteration period of a p-stage 1F1B pipeline in which stage s, at its
    bubble instruction k, does not proceed before waits[k] has passed since its previous
    instruction ended (Sec. 4.2: during profiling the engine holds back the instruction
    after a bubble instruction for a set time).  Plain dependency simulation: forward j of stage q needs
    forward j of stage q-1, backward j of stage q needs backward j of stage q+1, each stage
    runs its instructions in order, iterations follow each other without a gap.  Returns the
    time between the ends of the last two simulated iterations."""
    progs = [stage_program_1f1b(p, m, q) for q in range(p)]
    done_f = {}
    done_b = {}
    pc = [0] * p
    it = [0] * p
    free_at = [0] * p          # when the stage finished its previous instruction
    not_before = [0] * p       # earliest start imposed by a wait
    end_of_iter = [0] * iterations
    remaining = p * iterations
    while remaining:
        progressed = False
        for q in range(p):
            while it[q] < iterations:
                kind, idx = progs[q][pc[q]]
                if kind == "BUBBLE":
                    if q == s:
                        not_before[q] = free_at[q] + waits[idx]
                else:
                    if kind == "F":
                        dep = done_f.get((q - 1, idx, it[q])) if q > 0 else 0
                    else:
                        dep = done_b.get((q + 1, idx, it[q])) if q < p - 1 else 0
                    if dep is None:
                        break
                    start = max(free_at[q], not_before[q], dep)
                    end = start + (tf if kind == "F" else tb)
                    (done_f if kind == "F" else done_b)[(q, idx, it[q])] = end
                    free_at[q] = end
                    end_of_iter[it[q]] = max(end_of_iter[it[q]], end)
                progressed = True
                pc[q] += 1
                if pc[q] == len(progs[q]):
                    pc[q] = 0
                    it[q] += 1
                    remaining -= 1
        assert progressed, "dependency deadlock"
    return end_of_iter[-1] - end_of_iter[-2]


def probe_bubble_durations(p, m, s, tf, tb, first_wait, tol_ppm=0):
    """The doubling probe of Sec. 4.2.  The bubble instructions of stage s are characterised
    one after the other, in program order, the waits already found staying in place: wait
    first_wait at the instruction; while the iteration period stays within tol_ppm of the
    undisturbed one, double the wait; the estimate is the last wait that left the period
    unaffected (0 if even first_wait slowed the pipeline).  A wait may exceed the idle window
    it sits in when later windows of the stage absorb the delay (the pipeline only slows once
    the slack is used up); holding the earlier estimates makes the set jointly harmless.
    Returns one estimate per idle window of windows_1f1b(p, m, s, ...), in the same order."""
    n = sum(1 for ins in stage_program_1f1b(p, m, s) if ins[0] == "BUBBLE")
    base = pipeline_period_with_waits(p, m, tf, tb, s, [0] * n)
    limit = base + base * tol_ppm // 1_000_000
    waits = [0] * n
    for k in range(n):
        w = first_wait
        while True:
            trial = list(waits)
            trial[k] = w
            if pipeline_period_with_waits(p, m, tf, tb, s, trial) > limit:
                break
            waits[k] = w
            w *= 2
    return waits
