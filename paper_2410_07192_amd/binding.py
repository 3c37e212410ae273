"""ctypes binding of libpipefill.so: same names as the C ABI, argument marshalling only.

Every step of the path runs inside the library; this module converts Python values to the C
structs and back, and packs NumPy parameter dictionaries into the library's layer-blob layout.
There is no fallback: if the shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

# A context with streamed weights, offload or the timeline loop creates streams of its own next to the caller's;
# with HIP's default of four hardware queues per process some of them would share a queue and a copy would wait
# behind the kernels it is meant to overlap.  Only effective if the HIP runtime is not loaded yet (import this
# module, or set the variable, before torch).
if int(os.environ.get("GPU_MAX_HW_QUEUES", "4") or 4) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpipefill.so")

PF_OK, PF_ERR_ARG, PF_ERR_CAPACITY, PF_ERR_INFEASIBLE, PF_ERR_NOMEM, PF_ERR_HIP, PF_ERR_STATE = 0, -1, -2, -3, -4, -5, -6
PF_BUBBLE_FWD_BWD, PF_BUBBLE_GAP, PF_BUBBLE_FILL_DRAIN, PF_BUBBLE_EXPLICIT = 0, 1, 2, 3
PF_OP_EMBED, PF_OP_LAYER_FWD, PF_OP_FINAL_LN, PF_OP_HEAD_LOSS, PF_OP_LAYER_BWD, PF_OP_OPT = range(6)
PF_DTYPE_F32, PF_DTYPE_BF16 = 0, 1
PF_INSTR_FWD, PF_INSTR_BWD, PF_INSTR_BUBBLE, PF_INSTR_OPT = 0, 1, 2, 3
PF_POLICY_FIFO, PF_POLICY_SJF, PF_POLICY_MAKESPAN = 0, 1, 2

EXPORTS = [
    "pf_last_error", "pf_version", "pf_schedule_1f1b", "pf_schedule_gpipe", "pf_plan_bubbles", "pf_plan_bubbles_from", "pf_probe_bubbles", "pf_offload_plan", "pf_job_time", "pf_sched_simulate",
    "pf_select_config", "pf_build_chain", "pf_layer_blob_layout", "pf_ctx_arena_bytes", "pf_ctx_create",
    "pf_ctx_destroy", "pf_ctx_sync", "pf_ctx_set_io", "pf_load_layer_async", "pf_fill_chunk_fwd",
    "pf_fill_chunk_bwd", "pf_fill_chunk", "pf_profile_chain", "pf_main_stage_step", "pf_timeline_run",
    "pf_ctx_set_replan", "pf_main_opt_state_bytes", "pf_ctx_set_main_offload", "pf_ctx_kernel_timing_every", "pf_ctx_train_state", "pf_ctx_read_params", "pf_op_gemm", "pf_op_layernorm", "pf_op_attention",
    "pf_op_embed", "pf_ctx_kernel_timing", "pf_ctx_kernel_stats", "pf_op_attention_bwd", "pf_op_layernorm_bwd", "pf_op_transpose", "pf_op_gemm_tn",
    "pf_op_layernorm_bwd_static", "pf_select_config_stream", "pf_main_stage_read", "pf_probe_bubbles_live",
]
PF_K_GEMM_QKV, PF_K_GEMM_OUT, PF_K_GEMM_FFN1, PF_K_GEMM_FFN2, PF_K_ATTENTION, PF_K_LAYERNORM, PF_K_EMBED, PF_K_COPY_WAIT = range(8)


class PipeFillError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"pipefill error {code}: {msg}")
        self.code = code
        self.msg = msg


class pf_bubble(C.Structure):
    _fields_ = [("start_ns", C.c_int64), ("dur_ns", C.c_int64), ("free_bytes", C.c_int64),
                ("kind", C.c_int32), ("fillable", C.c_int32)]


class pf_node(C.Structure):
    _fields_ = [("dur_ns", C.c_int64), ("mem_bytes", C.c_int64), ("op", C.c_int32), ("layer", C.c_int32),
                ("mb_first", C.c_int32), ("mb_count", C.c_int32)]


class pf_chunk(C.Structure):
    _fields_ = [("bubble", C.c_int32), ("cycle", C.c_int32), ("node_begin", C.c_int32), ("node_end", C.c_int32),
                ("dur_ns", C.c_int64), ("mem_bytes", C.c_int64)]


class pf_job(C.Structure):
    _fields_ = [("arrival_ns", C.c_int64), ("deadline_ns", C.c_int64)]


class pf_job_run(C.Structure):
    _fields_ = [("start_ns", C.c_int64), ("finish_ns", C.c_int64), ("device", C.c_int32), ("reserved", C.c_int32)]


class pf_model_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ff", C.c_int32),
                ("seq_len", C.c_int32), ("batch", C.c_int32), ("vocab", C.c_int32), ("causal", C.c_int32),
                ("dtype", C.c_int32), ("eps", C.c_float)]


class pf_exec_config(C.Structure):
    _fields_ = [("g", C.c_int32), ("streamed", C.c_int32), ("n_slots", C.c_int32), ("training", C.c_int32)]


class pf_weights(C.Structure):
    _fields_ = [("layers", C.POINTER(C.c_void_p)), ("tok_emb", C.c_void_p), ("pos_emb", C.c_void_p),
                ("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p)]


class pf_adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("accum", C.c_int32)]


class pf_timeline_stats(C.Structure):
    _fields_ = [("iter_ns", C.c_int64), ("offered_ns", C.c_int64), ("idle_ns", C.c_int64),
                ("fill_busy_ns", C.c_int64), ("overrun_ns", C.c_int64), ("main_busy_ns", C.c_int64),
                ("chunks_run", C.c_int32), ("replicas_done", C.c_int32), ("offload_wait_ns", C.c_int64),
                ("offloaded_bytes", C.c_int64)]

    def asdict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_07192_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    lib.pf_last_error.restype = C.c_char_p
    lib.pf_layer_blob_layout.restype = C.c_int64
    lib.pf_ctx_arena_bytes.restype = C.c_int64
    I32, I64, VP = C.c_int32, C.c_int64, C.c_void_p
    P = C.POINTER
    lib.pf_schedule_1f1b.argtypes = [I32, I32, I32, I64, I64, I64, I32, I64, P(pf_bubble), I32, P(I32)]
    lib.pf_schedule_gpipe.argtypes = [I32, I32, I32, I64, I64, I64, P(pf_bubble), I32, P(I32)]
    lib.pf_plan_bubbles.argtypes = [P(pf_bubble), I32, P(pf_node), I32, I64, I64, I32, P(pf_chunk), I32, P(I32), P(I32)]
    lib.pf_job_time.argtypes = [P(pf_bubble), I32, P(pf_node), I32, I64, I64, I64, I64, I64, P(I64)]
    lib.pf_sched_simulate.argtypes = [I32, P(pf_job), I32, I32, P(I64), P(pf_job_run), P(I64), P(I64)]
    lib.pf_probe_bubbles.argtypes = [I32, I32, I32, I64, I64, I64, I64, P(I64), I32, P(I32)]
    lib.pf_offload_plan.argtypes = [I32, I32, I32, I64, I64, I64, I64, I64, P(I64), P(I64), I32, P(I32)]
    lib.pf_plan_bubbles_from.argtypes = [P(pf_bubble), I32, P(pf_node), I32, I64, I64, I32, I64, P(pf_chunk), I32, P(I32),
                                         P(I32)]
    lib.pf_select_config_stream.argtypes = [P(pf_bubble), I32, P(P(pf_node)), P(I32), P(I64), I32, I64, I64, I32, I32,
                                            P(I32), P(I32), P(I32), P(I32)]
    lib.pf_select_config.argtypes = [P(pf_bubble), I32, P(P(pf_node)), P(I32), P(I64), I32, I64, I64, I32,
                                     P(I32), P(I32), P(I32), P(I32)]
    lib.pf_build_chain.argtypes = [P(pf_model_desc), P(pf_exec_config), P(pf_node), I32, P(I32)]
    lib.pf_layer_blob_layout.argtypes = [P(pf_model_desc), P(I64)]
    lib.pf_ctx_arena_bytes.argtypes = [P(pf_model_desc), P(pf_exec_config)]
    lib.pf_ctx_create.argtypes = [P(pf_model_desc), P(pf_exec_config), P(pf_weights), P(pf_adam), VP, I64, P(VP)]
    lib.pf_ctx_destroy.argtypes = [VP]
    lib.pf_ctx_sync.argtypes = [VP]
    lib.pf_ctx_set_io.argtypes = [VP, VP, I32, VP, I32]
    lib.pf_load_layer_async.argtypes = [VP, I32, I32, VP]
    lib.pf_fill_chunk_fwd.argtypes = [VP, P(pf_chunk), P(pf_node), I32, VP, VP, I64, VP]
    lib.pf_fill_chunk_bwd.argtypes = [VP, P(pf_chunk), P(pf_node), I32, VP, VP, I64, VP]
    lib.pf_fill_chunk.argtypes = [VP, P(pf_chunk), P(pf_node), I32, I64, VP]
    lib.pf_profile_chain.argtypes = [VP, P(pf_node), I32, I32, I32, VP]
    lib.pf_main_stage_step.argtypes = [VP, I32, I32, VP, VP]
    lib.pf_probe_bubbles_live.argtypes = [VP, VP, I32, I32, I32, I64, I64, I64, I64, P(I64), I32, P(I32), P(I64), VP]
    lib.pf_main_stage_read.argtypes = [VP, I32, I32, VP, I64, VP]
    lib.pf_timeline_run.argtypes = [VP, VP, VP, I32, I32, I32, I64, I64, P(pf_bubble), I32, P(pf_chunk), I32,
                                    P(pf_node), I32, P(I32), VP, VP, P(pf_timeline_stats)]
    lib.pf_ctx_set_replan.argtypes = [VP, I32, I64, I64]
    lib.pf_main_opt_state_bytes.argtypes = [VP, P(I64)]
    lib.pf_ctx_set_main_offload.argtypes = [VP, I64, VP, I64, P(I64), I32, I32]
    lib.pf_ctx_kernel_timing_every.argtypes = [VP, I32]
    lib.pf_ctx_train_state.argtypes = [VP, P(C.c_double), P(I64)]
    lib.pf_ctx_read_params.argtypes = [VP, I32, I32, VP, I64, VP]
    lib.pf_ctx_kernel_timing.argtypes = [VP, C.c_uint32]
    lib.pf_ctx_kernel_stats.argtypes = [VP, I32, P(I64), P(I64)]
    lib.pf_op_gemm.argtypes = [I32, VP, VP, VP, I64, I64, I64, VP, VP, I32, I32, I32, VP, VP, VP]
    lib.pf_op_layernorm.argtypes = [I32, VP, VP, VP, VP, VP, VP, I64, I32, C.c_float, VP, I64, VP]
    lib.pf_op_attention.argtypes = [I32, VP, VP, VP, I32, I32, I32, I32, I32, VP]
    lib.pf_op_attention_bwd.argtypes = [I32, VP, VP, VP, VP, VP, VP, I32, I32, I32, I32, I32, VP]
    lib.pf_op_layernorm_bwd.argtypes = [I32, VP, VP, VP, VP, VP, VP, VP, VP, VP, VP, I64, I32, VP]
    lib.pf_op_layernorm_bwd_static.argtypes = [I32, VP, VP, VP, VP, VP, VP, VP, VP, VP, I64, I32, VP]
    lib.pf_op_transpose.argtypes = [I32, VP, VP, I64, I64, VP, VP]
    lib.pf_op_gemm_tn.argtypes = [I32, VP, VP, VP, VP, I64, I64, I64, VP]
    lib.pf_op_embed.argtypes = [I32, VP, VP, VP, VP, I64, I32, I32, I32, VP]
    return lib


lib = _load()


def _check(rc):
    if rc != PF_OK:
        raise PipeFillError(rc, lib.pf_last_error().decode())


# ------------------------------------------------------------------------------------------ planner
def _bubble_dict(b):
    return dict(start=b.start_ns, dur=b.dur_ns, free=b.free_bytes, kind=b.kind, fillable=b.fillable)


def bubbles_to_c(bubbles):
    arr = (pf_bubble * max(1, len(bubbles)))()
    for i, b in enumerate(bubbles):
        arr[i] = pf_bubble(b.get("start", 0), b["dur"], b["free"], b.get("kind", PF_BUBBLE_EXPLICIT),
                           b.get("fillable", 1))
    return arr


def nodes_to_c(F):
    """F: list of (dur, mem) or (dur, mem, op, layer, mb_first, mb_count) tuples, or pf_node array."""
    if isinstance(F, C.Array):
        return F
    arr = (pf_node * max(1, len(F)))()
    for i, n in enumerate(F):
        n = tuple(n)
        if len(n) == 2:
            n = n + (PF_OP_LAYER_FWD, 0, 0, 1)
        arr[i] = pf_node(*n)
    return arr


def pf_schedule_1f1b(p, m, stage, tf_ns, tb_ns, free_bytes, fill_gaps=True, min_window_ns=0, cap=None):
    cap = (m + 2) if cap is None else cap
    out = (pf_bubble * max(1, cap))()
    n = C.c_int32(0)
    _check(lib.pf_schedule_1f1b(p, m, stage, tf_ns, tb_ns, free_bytes, int(bool(fill_gaps)), min_window_ns,
                                out, cap, C.byref(n)))
    return [_bubble_dict(out[i]) for i in range(n.value)]


def pf_schedule_gpipe(p, m, stage, tf_ns, tb_ns, free_bytes, cap=2):
    out = (pf_bubble * max(1, cap))()
    n = C.c_int32(0)
    _check(lib.pf_schedule_gpipe(p, m, stage, tf_ns, tb_ns, free_bytes, out, cap, C.byref(n)))
    return [_bubble_dict(out[i]) for i in range(n.value)]


def pf_job_time(bubbles, F, samples_per_replica, total_samples, iter_ns, fill_ppm=1_000_000, switch_ns=0):
    t = C.c_int64(0)
    _check(lib.pf_job_time(bubbles_to_c(bubbles), len(bubbles), nodes_to_c(F), len(F), samples_per_replica,
                           total_samples, iter_ns, fill_ppm, switch_ns, C.byref(t)))
    return t.value


def pf_sched_simulate(policy, jobs, proc, n_dev):
    """jobs: list of dicts (arrival[, deadline]); proc[j][i].  Returns ([(device, start, finish)], makespan, sum)."""
    n = len(jobs)
    cj = (pf_job * max(1, n))()
    for i, j in enumerate(jobs):
        cj[i].arrival_ns = j["arrival"]
        cj[i].deadline_ns = j.get("deadline", -1)
    flat = (C.c_int64 * max(1, n * n_dev))(*[proc[j][d] for j in range(n) for d in range(n_dev)])
    runs = (pf_job_run * max(1, n))()
    mk, sm = C.c_int64(0), C.c_int64(0)
    _check(lib.pf_sched_simulate(policy, cj, n, n_dev, flat, runs, C.byref(mk), C.byref(sm)))
    return [(runs[i].device, runs[i].start_ns, runs[i].finish_ns) for i in range(n)], mk.value, sm.value


def pf_probe_bubbles(p, m, stage, tf_ns, tb_ns, first_wait_ns, tol_ppm=0):
    """Estimated harmless wait per idle window of the stage (doubling probe)."""
    n = C.c_int32(0)
    rc = lib.pf_probe_bubbles(p, m, stage, tf_ns, tb_ns, first_wait_ns, tol_ppm, None, 0, C.byref(n))
    if rc not in (PF_OK, PF_ERR_CAPACITY):
        raise PipeFillError(rc, lib.pf_last_error().decode())
    out = (C.c_int64 * max(1, n.value))()
    _check(lib.pf_probe_bubbles(p, m, stage, tf_ns, tb_ns, first_wait_ns, tol_ppm, out, n.value, C.byref(n)))
    return [int(out[i]) for i in range(n.value)]


def pf_probe_bubbles_live(main_ctx, main_io, p, m, stage, tf_ns, tb_ns, first_wait_ns, tol_ppm, stream=None):
    """The doubling probe with the stage's instructions run on the device.  Returns (estimates, undisturbed period)."""
    n = C.c_int32(0)
    out = (C.c_int64 * (m + 2))()
    base = C.c_int64(0)
    _check(lib.pf_probe_bubbles_live(main_ctx.handle, main_io, p, m, stage, tf_ns, tb_ns, first_wait_ns, tol_ppm, out,
                                     m + 2, C.byref(n), C.byref(base), stream))
    return [int(out[i]) for i in range(n.value)], int(base.value)


def pf_offload_plan(p, m, stage, tf_ns, sync_ns, state_bytes, d2h_bytes_per_s, h2d_bytes_per_s):
    """(bytes leaving with each forward, bytes off the device in each idle window of the stage)."""
    n = C.c_int32(0)
    sl = (C.c_int64 * max(1, m))()
    rc = lib.pf_offload_plan(p, m, stage, tf_ns, sync_ns, state_bytes, d2h_bytes_per_s, h2d_bytes_per_s, sl, None, 0,
                             C.byref(n))
    if rc not in (PF_OK, PF_ERR_CAPACITY):
        raise PipeFillError(rc, lib.pf_last_error().decode())
    ex = (C.c_int64 * max(1, n.value))()
    _check(lib.pf_offload_plan(p, m, stage, tf_ns, sync_ns, state_bytes, d2h_bytes_per_s, h2d_bytes_per_s, sl, ex,
                               n.value, C.byref(n)))
    return [int(sl[j]) for j in range(m)], [int(ex[k]) for k in range(n.value)]


def pf_plan_bubbles(bubbles, F, fill_ppm=1_000_000, switch_ns=0, first_bubble=0, cap=None, raw=False,
                    first_dur_ns=-1):
    """Returns (chunks, replicas); chunks as dicts, or as the ctypes array and count when raw.
    first_dur_ns >= 0 plans through pf_plan_bubbles_from (first visit of the first bubble shortened)."""
    B = bubbles_to_c(bubbles)
    Fc = nodes_to_c(F)
    nF = len(F)
    n = C.c_int32(0)
    k = C.c_int32(0)
    if cap is None:
        rc = lib.pf_plan_bubbles_from(B, len(bubbles), Fc, nF, fill_ppm, switch_ns, first_bubble, first_dur_ns,
                                      None, 0, C.byref(n), C.byref(k))
        if rc not in (PF_OK, PF_ERR_CAPACITY):
            e = PipeFillError(rc, lib.pf_last_error().decode())
            e.node = n.value
            raise e
        cap = n.value
    out = (pf_chunk * max(1, cap))()
    if first_dur_ns < 0:
        rc = lib.pf_plan_bubbles(B, len(bubbles), Fc, nF, fill_ppm, switch_ns, first_bubble, out, cap,
                                 C.byref(n), C.byref(k))
    else:
        rc = lib.pf_plan_bubbles_from(B, len(bubbles), Fc, nF, fill_ppm, switch_ns, first_bubble, first_dur_ns,
                                      out, cap, C.byref(n), C.byref(k))
    if rc != PF_OK:
        e = PipeFillError(rc, lib.pf_last_error().decode())
        e.node = n.value
        e.needed = n.value
        raise e
    if raw:
        return out, n.value, k.value
    chunks = [dict(bubble=c.bubble, cycle=c.cycle, node_begin=c.node_begin, node_end=c.node_end,
                   dur=c.dur_ns, mem=c.mem_bytes) for c in out[:n.value]]
    return chunks, k.value


def pf_select_config(bubbles, configs, fill_ppm=1_000_000, switch_ns=0, first_bubble=0):
    """configs: list of dicts (F, samples).  Returns (best, replicas[], cycles[], chunks[])."""
    B = bubbles_to_c(bubbles)
    n = len(configs)
    keep = [nodes_to_c(c["F"]) for c in configs]
    chains = (C.POINTER(pf_node) * n)(*[C.cast(a, C.POINTER(pf_node)) for a in keep])
    nn = (C.c_int32 * n)(*[len(c["F"]) for c in configs])
    samples = (C.c_int64 * n)(*[c["samples"] for c in configs])
    best = C.c_int32(-1)
    rep = (C.c_int32 * n)()
    cyc = (C.c_int32 * n)()
    chk = (C.c_int32 * n)()
    rc = lib.pf_select_config(B, len(bubbles), chains, nn, samples, n, fill_ppm, switch_ns, first_bubble,
                              C.byref(best), rep, cyc, chk)
    if rc == PF_ERR_INFEASIBLE:
        return -1, list(rep), list(cyc), list(chk)
    _check(rc)
    return best.value, list(rep), list(cyc), list(chk)


def pf_select_config_stream(bubbles, configs, fill_ppm=1_000_000, switch_ns=0, first_bubble=0, horizon_cycles=8):
    """configs: list of dicts (F, samples).  Returns (best, runs[], cycles[], chunks[])."""
    B = bubbles_to_c(bubbles)
    n = len(configs)
    keep = [nodes_to_c(c["F"]) for c in configs]
    chains = (C.POINTER(pf_node) * n)(*[C.cast(a, C.POINTER(pf_node)) for a in keep])
    nn = (C.c_int32 * n)(*[len(c["F"]) for c in configs])
    samples = (C.c_int64 * n)(*[c["samples"] for c in configs])
    best = C.c_int32(-1)
    runs = (C.c_int32 * n)()
    cyc = (C.c_int32 * n)()
    chk = (C.c_int32 * n)()
    rc = lib.pf_select_config_stream(B, len(bubbles), chains, nn, samples, n, fill_ppm, switch_ns, first_bubble,
                                     horizon_cycles, C.byref(best), runs, cyc, chk)
    if rc == PF_ERR_INFEASIBLE:
        return -1, list(runs), list(cyc), list(chk)
    _check(rc)
    return best.value, list(runs), list(cyc), list(chk)


# ------------------------------------------------------------------------------------------ model
def model_desc(shape, batch=None):
    """shape: synth.ModelShape (or anything with the same attributes)."""
    return pf_model_desc(shape.n_layers, shape.d_model, shape.n_heads, shape.d_ff, shape.seq_len,
                         shape.batch if batch is None else batch, shape.vocab, int(shape.causal),
                         PF_DTYPE_BF16 if shape.dtype == "bf16" else PF_DTYPE_F32, shape.eps)


def pf_layer_blob_layout(md):
    off = (C.c_int64 * 12)()
    size = lib.pf_layer_blob_layout(C.byref(md), off)
    if size < 0:
        _check(int(size))
    return int(size), list(off)


def pf_ctx_arena_bytes(md, cfg):
    n = lib.pf_ctx_arena_bytes(C.byref(md), C.byref(cfg))
    if n < 0:
        _check(int(n))
    return int(n)


def pf_build_chain(md, cfg, cap=None):
    cap = (2 * md.n_layers + 8) if cap is None else cap
    out = (pf_node * max(1, cap))()
    n = C.c_int32(0)
    _check(lib.pf_build_chain(C.byref(md), C.byref(cfg), out, cap, C.byref(n)))
    arr = (pf_node * n.value)()
    for i in range(n.value):
        arr[i] = out[i]
    return arr


def f32_to_bf16_bits(a):
    """float32 array -> uint16 bf16 bit patterns (values are expected to be bf16-representable already;
    rounding to nearest even otherwise)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> 16) & 1))) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


_BLOB_ORDER = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def pack_layer_blob(md, params, out=None):
    """Layer parameters ([in, out] matrices, float32) -> one packed host blob (uint8) in the
    library's layout: matrices transposed to [out, in], elements in the model dtype."""
    size, off = pf_layer_blob_layout(md)
    blob = np.zeros(size, dtype=np.uint8) if out is None else out
    bf16 = md.dtype == PF_DTYPE_BF16
    for i, name in enumerate(_BLOB_ORDER):
        a = np.asarray(params[name], dtype=np.float32)
        if a.ndim == 2:
            a = np.ascontiguousarray(a.T)
        raw = f32_to_bf16_bits(a).view(np.uint8) if bf16 else np.ascontiguousarray(a).view(np.uint8)
        raw = raw.reshape(-1)
        blob[off[i]:off[i] + raw.size] = raw
    return blob


def to_storage(a, md):
    """float32 array -> array in the model's storage dtype (uint16 bf16 bits or float32)."""
    return f32_to_bf16_bits(a) if md.dtype == PF_DTYPE_BF16 else np.ascontiguousarray(a, dtype=np.float32)


def from_storage(a, md):
    return bf16_bits_to_f32(a) if md.dtype == PF_DTYPE_BF16 else np.asarray(a, dtype=np.float32)


# ------------------------------------------------------------------------------------------ context
class Context:
    """Owns a pf_ctx handle.  Pointers are plain integers (e.g. torch.Tensor.data_ptr())."""

    def __init__(self, md, cfg, layer_ptrs, tok_emb, pos_emb, lnf_g, lnf_b, arena_ptr, arena_bytes, adam=None):
        self.md, self.cfg = md, cfg
        self._layers = (C.c_void_p * md.n_layers)(*layer_ptrs)
        w = pf_weights(C.cast(self._layers, C.POINTER(C.c_void_p)), tok_emb, pos_emb, lnf_g, lnf_b)
        h = C.c_void_p(None)
        _check(lib.pf_ctx_create(C.byref(md), C.byref(cfg), C.byref(w), C.byref(adam) if adam else None,
                                 arena_ptr, arena_bytes, C.byref(h)))
        self.handle = h

    def destroy(self):
        if self.handle:
            lib.pf_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def pf_ctx_sync(self):
        _check(lib.pf_ctx_sync(self.handle))

    def pf_ctx_set_io(self, in_ptr, n_in, out_ptr, n_out):
        _check(lib.pf_ctx_set_io(self.handle, in_ptr, n_in, out_ptr, n_out))

    def pf_load_layer_async(self, layer, slot, copy_stream=None):
        _check(lib.pf_load_layer_async(self.handle, layer, slot, copy_stream))

    def pf_fill_chunk_fwd(self, chunk, F, act_in=None, act_out=None, cap_bytes=0, stream=None):
        _check(lib.pf_fill_chunk_fwd(self.handle, C.byref(chunk), F, len(F), act_in, act_out, cap_bytes, stream))

    def pf_fill_chunk_bwd(self, chunk, F, grad_io=None, grad_out=None, cap_bytes=0, stream=None):
        _check(lib.pf_fill_chunk_bwd(self.handle, C.byref(chunk), F, len(F), grad_io, grad_out, cap_bytes, stream))

    def pf_fill_chunk(self, chunk, F, cap_bytes=0, stream=None):
        _check(lib.pf_fill_chunk(self.handle, C.byref(chunk), F, len(F), cap_bytes, stream))

    def pf_profile_chain(self, F, warmup=2, reps=5, stream=None):
        _check(lib.pf_profile_chain(self.handle, F, len(F), warmup, reps, stream))

    def pf_main_stage_step(self, instr, index, io_ptr, stream=None):
        _check(lib.pf_main_stage_step(self.handle, instr, index, io_ptr, stream))

    def pf_main_stage_read(self, what, index, dst, dst_bytes, stream=None):
        _check(lib.pf_main_stage_read(self.handle, what, index, dst, dst_bytes, stream))

    def pf_ctx_kernel_timing(self, mask):
        _check(lib.pf_ctx_kernel_timing(self.handle, mask))

    def pf_ctx_kernel_stats(self, cls):
        n = C.c_int64(0)
        t = C.c_int64(0)
        _check(lib.pf_ctx_kernel_stats(self.handle, cls, C.byref(n), C.byref(t)))
        return n.value, t.value

    def pf_ctx_kernel_timing_every(self, n):
        _check(lib.pf_ctx_kernel_timing_every(self.handle, n))

    def pf_ctx_set_replan(self, enable, fill_ppm=1000000, switch_ns=0):
        _check(lib.pf_ctx_set_replan(self.handle, int(bool(enable)), fill_ppm, switch_ns))

    def pf_ctx_train_state(self):
        loss = C.c_double(0.0)
        steps = C.c_int64(0)
        _check(lib.pf_ctx_train_state(self.handle, C.byref(loss), C.byref(steps)))
        return loss.value, steps.value

    def pf_main_opt_state_bytes(self):
        n = C.c_int64(0)
        _check(lib.pf_main_opt_state_bytes(self.handle, C.byref(n)))
        return n.value

    def pf_ctx_set_main_offload(self, sync_ns, host_ptr=None, host_bytes=0, slice_bytes=(), scrub=False):
        n = len(slice_bytes)
        arr = (C.c_int64 * max(1, n))(*slice_bytes)
        _check(lib.pf_ctx_set_main_offload(self.handle, sync_ns, host_ptr, host_bytes, arr, n, int(bool(scrub))))

    def pf_ctx_read_params(self, what, layer, dst_ptr, dst_bytes, stream=None):
        _check(lib.pf_ctx_read_params(self.handle, what, layer, dst_ptr, dst_bytes, stream))


def pf_timeline_run(fill_ctx, main_ctx, main_io, p, m, stage, tf_ns, tb_ns, windows, plan, n_plan, F, cursor,
                    fill_stream, main_stream):
    """windows: list of dicts or pf_bubble array; plan: pf_chunk array; cursor: ctypes c_int32 (in/out)."""
    W = windows if isinstance(windows, C.Array) else bubbles_to_c(windows)
    nW = len(windows)
    st = pf_timeline_stats()
    _check(lib.pf_timeline_run(fill_ctx.handle if fill_ctx else None, main_ctx.handle if main_ctx else None,
                               main_io, p, m, stage, tf_ns, tb_ns, W, nW, plan, n_plan, F,
                               len(F) if F is not None else 0, C.byref(cursor), fill_stream, main_stream,
                               C.byref(st)))
    return st.asdict()


# ------------------------------------------------------------------------------------------ kernels
def pf_op_gemm(dtype, X, W, Cp, M, N, K, bias=None, resid=None, gelu=0, out_f32=0, accumulate=0, stream=None, dact_in=None,
               preact_out=None):
    _check(lib.pf_op_gemm(dtype, X, W, Cp, M, N, K, bias, resid, gelu, out_f32, accumulate, dact_in, preact_out, stream))


def pf_op_layernorm(dtype, x, g, b, y, rows, d, eps, mean_out=None, rstd_out=None, stream=None, warm=None, warm_bytes=0):
    _check(lib.pf_op_layernorm(dtype, x, g, b, y, mean_out, rstd_out, rows, d, eps, warm, warm_bytes, stream))


def pf_op_attention(dtype, qkv, out, B, S, h, dh, causal, lse=None, stream=None):
    _check(lib.pf_op_attention(dtype, qkv, out, lse, B, S, h, dh, int(bool(causal)), stream))


def pf_op_embed(dtype, ids, tok, pos, x, tokens, S, d, V, stream=None):
    _check(lib.pf_op_embed(dtype, ids, tok, pos, x, tokens, S, d, V, stream))


def unpack_layer_blob_f32(md, raw):
    """fp32 layer blob as returned by pf_ctx_read_params (uint8 or float32 array) -> dict of float32 arrays
    in the mathematical layout ([in, out] matrices)."""
    md32 = pf_model_desc.from_buffer_copy(md)
    md32.dtype = PF_DTYPE_F32
    size, off = pf_layer_blob_layout(md32)
    raw = np.ascontiguousarray(raw).view(np.uint8).reshape(-1)
    d, f = md.d_model, md.d_ff
    shapes = {"ln1_g": (d,), "ln1_b": (d,), "w_qkv": (3 * d, d), "b_qkv": (3 * d,), "w_o": (d, d), "b_o": (d,),
              "ln2_g": (d,), "ln2_b": (d,), "w_1": (f, d), "b_1": (f,), "w_2": (d, f), "b_2": (d,)}
    out = {}
    for i, name in enumerate(_BLOB_ORDER):
        n = int(np.prod(shapes[name]))
        a = raw[off[i]:off[i] + 4 * n].view(np.float32).reshape(shapes[name])
        out[name] = a.T.copy() if a.ndim == 2 else a.copy()
    return out, size


def unpack_embedding_f32(md, raw):
    """fp32 tok | pos | lnf_g | lnf_b block of pf_ctx_read_params(layer=-1) -> dict."""
    raw = np.ascontiguousarray(raw).view(np.uint8).reshape(-1)
    al = lambda x: (x + 255) // 256 * 256
    vp = (md.vocab + 63) // 64 * 64
    d, S = md.d_model, md.seq_len
    o1 = al(vp * d * 4)
    o2 = o1 + al(S * d * 4)
    o3 = o2 + al(d * 4)
    total = o3 + al(d * 4)
    tok = raw[0:vp * d * 4].view(np.float32).reshape(vp, d)
    return dict(tok_emb=tok[:md.vocab].copy(), tok_pad=tok[md.vocab:].copy(),
                pos_emb=raw[o1:o1 + S * d * 4].view(np.float32).reshape(S, d).copy(),
                lnf_g=raw[o2:o2 + d * 4].view(np.float32).copy(),
                lnf_b=raw[o3:o3 + d * 4].view(np.float32).copy()), total


def pf_op_layernorm_bwd(dtype, dy, x, g, mean, rstd, resid, dx, dg, db, partial, rows, d, stream=None):
    _check(lib.pf_op_layernorm_bwd(dtype, dy, x, g, mean, rstd, resid, dx, dg, db, partial, rows, d, stream))


def pf_op_layernorm_bwd_static(dtype, dy, x, g, mean, rstd, resid, dx, dg, db, rows, d, stream=None):
    _check(lib.pf_op_layernorm_bwd_static(dtype, dy, x, g, mean, rstd, resid, dx, dg, db, rows, d, stream))


def pf_op_gemm_tn(dtype, A, B, Cp, M, N, K, colsum_acc=None, stream=None):
    _check(lib.pf_op_gemm_tn(dtype, A, B, Cp, colsum_acc, M, N, K, stream))


def pf_op_transpose(dtype, src, dst, rows, cols, colsum_acc=None, stream=None):
    _check(lib.pf_op_transpose(dtype, src, dst, rows, cols, colsum_acc, stream))


def pf_op_attention_bwd(dtype, qkv, out, dout, lse, dsum, dqkv, B, S, h, dh, causal, stream=None):
    _check(lib.pf_op_attention_bwd(dtype, qkv, out, dout, lse, dsum, dqkv, B, S, h, dh, int(bool(causal)), stream))
