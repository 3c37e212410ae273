/*
 * pipefill.h -- C ABI of the MI355X (gfx950) fill-job Executor library.
 *
 * The library implements the bubble-bounded work of a fill-job Executor (Sec. 4.3 of the
 * PipeFill paper, arXiv 2410.07192): deriving the idle windows of a pipeline stage, partitioning
 * a fill job's linearised graph onto the bubble cycle (Algorithm 1), and executing one partition
 * ("chunk") of transformer-layer work per bubble with hand-written HIP kernels, optionally with
 * layer weights streamed from pinned host memory.  One emulated main-job stage provides the
 * bubbles (Sec. 4.2, the pipeline bubble instruction).
 *
 * Conventions
 *   - every call returns int32_t: PF_OK (0) or a negative PF_ERR_* code; nothing throws or aborts
 *     across this boundary; pf_last_error() returns a thread-local message for the last failure.
 *   - all times are int64 nanoseconds, all sizes int64 bytes, fractions are parts per million.
 *   - "host" / "device" in a parameter comment says where the pointed-to memory must live.
 *   - the caller owns every buffer it passes in; the library owns only what pf_ctx_create
 *     carves out of the caller's arena plus the streams/events it creates, released by
 *     pf_ctx_destroy.
 *   - streams are hipStream_t values passed as void* (NULL = the null stream).  Calls that take
 *     a stream enqueue work and return; only pf_ctx_sync, pf_profile_chain and pf_timeline_run
 *     wait for the device.
 *   - a context with streamed weights creates one copy stream, one with main-job offload one more,
 *     and pf_timeline_run one for its deadline stamps, next to the caller's fill and main streams.
 *     HIP gives a process four hardware queues unless GPU_MAX_HW_QUEUES says otherwise (read when
 *     the HIP runtime is loaded); streams beyond that share a queue, and a weight copy that shares
 *     the fill stream's queue waits behind the kernels it is meant to overlap (measured: a layer
 *     visit 1.7 ms longer, the whole copy).  Run with GPU_MAX_HW_QUEUES=8 or more.
 *   - a missing or failing GPU is an error (PF_ERR_HIP); there is no CPU fallback.
 */
#ifndef PIPEFILL_H
#define PIPEFILL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  PF_OK = 0,
  PF_ERR_ARG = -1,        /* null pointer, negative size, value out of range                     */
  PF_ERR_CAPACITY = -2,   /* output array too small; the needed count is written to *n_out       */
  PF_ERR_INFEASIBLE = -3, /* some graph node fits no bubble of the cycle                         */
  PF_ERR_NOMEM = -4,      /* arena too small / chunk exceeds the bubble's memory cap             */
  PF_ERR_HIP = -5,        /* a HIP runtime call failed (message in pf_last_error)                */
  PF_ERR_STATE = -6       /* call not valid in the context's current state                       */
};

/* kinds of idle window of one pipeline stage (Sec. 4.5, "Main job pipeline schedule") */
enum { PF_BUBBLE_FWD_BWD = 0, PF_BUBBLE_GAP = 1, PF_BUBBLE_FILL_DRAIN = 2, PF_BUBBLE_EXPLICIT = 3 };

/* graph-node operations of a transformer fill job */
enum { PF_OP_EMBED = 0, PF_OP_LAYER_FWD = 1, PF_OP_FINAL_LN = 2, PF_OP_HEAD_LOSS = 3,
       PF_OP_LAYER_BWD = 4, PF_OP_OPT = 5 };

enum { PF_DTYPE_F32 = 0, PF_DTYPE_BF16 = 1 };

/* kernel classes of a layer visit, for pf_ctx_kernel_timing / pf_ctx_kernel_stats.  PF_K_COPY_WAIT is no
 * kernel: it brackets the point where the fill stream waits for a streamed layer's host-to-HBM copy, so its
 * total is the time the fill stream sat idle inside its chunks because weights had not arrived. */
enum { PF_K_GEMM_QKV = 0, PF_K_GEMM_OUT = 1, PF_K_GEMM_FFN1 = 2, PF_K_GEMM_FFN2 = 3, PF_K_ATTENTION = 4,
       PF_K_LAYERNORM = 5, PF_K_EMBED = 6, PF_K_COPY_WAIT = 7, PF_KERNEL_CLASSES = 16 };

/* instructions of the emulated main-job stage (Sec. 4.2: forward / backward of a microbatch,
 * and the pipeline bubble instruction) */
enum { PF_INSTR_FWD = 0, PF_INSTR_BWD = 1, PF_INSTR_BUBBLE = 2, PF_INSTR_OPT = 3 };

/* One bubble of the cycle that repeats every main-job iteration (the lists B and M of
 * Algorithm 1): start relative to the global iteration start, duration, free HBM. */
typedef struct pf_bubble {
  int64_t start_ns;
  int64_t dur_ns;
  int64_t free_bytes;
  int32_t kind;      /* PF_BUBBLE_*                                                   */
  int32_t fillable;  /* 0: the planner skips this window                              */
} pf_bubble;

/* One node of the linearised graph (the list F of Algorithm 1): duration and peak memory
 * under one configuration, plus what it computes. */
typedef struct pf_node {
  int64_t dur_ns;
  int64_t mem_bytes;
  int32_t op;        /* PF_OP_*                                                       */
  int32_t layer;     /* layer index for LAYER_FWD / LAYER_BWD, else -1                */
  int32_t mb_first;  /* first fill microbatch of the visit                            */
  int32_t mb_count;  /* microbatches processed by this node (g per layer visit)       */
} pf_node;

/* One partition P[i] of Algorithm 1: nodes [node_begin, node_end) of the replicated chain
 * (node j is F[j mod nF] of replica j div nF) run in bubble `bubble` of cycle `cycle`. */
typedef struct pf_chunk {
  int32_t bubble;
  int32_t cycle;
  int32_t node_begin;
  int32_t node_end;
  int64_t dur_ns;    /* sum of node durations                                         */
  int64_t mem_bytes; /* max of node memory requirements                               */
} pf_chunk;

typedef struct pf_model_desc {
  int32_t n_layers, d_model, n_heads, d_ff, seq_len;
  int32_t batch;     /* sequences per fill microbatch                                 */
  int32_t vocab;     /* 0: hidden states are the input, no embedding / head           */
  int32_t causal;    /* 1: key j > query i is masked                                  */
  int32_t dtype;     /* PF_DTYPE_*: storage type of weights and activations           */
  float eps;         /* LayerNorm epsilon                                             */
} pf_model_desc;

/* One execution configuration of a job (Sec. 4.3: batch size x execution technique). */
typedef struct pf_exec_config {
  int32_t g;         /* microbatches per layer visit (>= 1)                           */
  int32_t streamed;  /* 1: layer weights live in pinned host memory                   */
  int32_t n_slots;   /* HBM weight slots when streamed (>= 2)                         */
  int32_t training;  /* 1: forward + recompute/backward + Adam                        */
} pf_exec_config;

/* Where the model's parameters live.  A layer is one packed blob (see pf_layer_blob_layout).
 * layers[l]: device pointer when the configuration is resident, pinned host pointer when it is
 * streamed.  tok_emb [vocab,d], pos_emb [seq,d], lnf_g [d], lnf_b [d]: device, model dtype;
 * the embeddings may be NULL when vocab == 0. */
typedef struct pf_weights {
  void* const* layers;   /* host array of n_layers pointers */
  void* tok_emb;
  void* pos_emb;
  void* lnf_g;
  void* lnf_b;
} pf_weights;

/* Adam constants for training fill jobs (the optimizer the paper names, Sec. 5). */
typedef struct pf_adam {
  float lr, beta1, beta2, eps;
  int32_t accum;     /* microbatches accumulated per optimizer step */
} pf_adam;

typedef struct pf_ctx pf_ctx;

/* ---- diagnostics ------------------------------------------------------------------------- */
const char* pf_last_error(void);           /* thread-local, never NULL                          */
int32_t pf_version(void);

/* ---- bubble windows (Sec. 2.1 idle fraction (p-1)/(m+p-1); Sec. 4.5 bubble lengths) -------- */
/* Idle windows of 0-based stage `stage` in one steady-state iteration of a 1F1B schedule with p
 * stages, m microbatches, forward/backward times tf_ns/tb_ns and zero communication time, in
 * time order: the fwd-bwd bubble of (p-s-1)*t_b + max(0,p-s-m)*t_f, the t_f-long non-contiguous
 * gaps before the cool-down backwards, the fill-drain bubble of s*(t_f+t_b).  Gaps get
 * fillable=1 only if fill_gaps != 0 and they last >= min_window_ns; contiguous bubbles always.
 * out: host array of `cap` entries; *n_out receives the count (also on PF_ERR_CAPACITY). */
int32_t pf_schedule_1f1b(int32_t p, int32_t m, int32_t stage, int64_t tf_ns, int64_t tb_ns,
                         int64_t free_bytes, int32_t fill_gaps, int64_t min_window_ns,
                         pf_bubble* out, int32_t cap, int32_t* n_out);
/* Same for GPipe: fwd-bwd bubble (p-s-1)*(t_f+t_b) and the identical fill-drain bubble. */
int32_t pf_schedule_gpipe(int32_t p, int32_t m, int32_t stage, int64_t tf_ns, int64_t tb_ns,
                          int64_t free_bytes, pf_bubble* out, int32_t cap, int32_t* n_out);

/* ---- Algorithm 1 (Sec. 4.3): partition a fill job onto the bubble cycle ------------------- */
/* B: host, the cycle (nB entries; entries with fillable==0 are skipped).  F: host, nF nodes.
 * Each bubble's usable duration is floor(dur*fill_ppm/1e6) - switch_ns, not below 0 (the
 * fill-fraction knob of Sec. 6.1).  The chain is replicated while one more copy keeps the total
 * strictly below the summed usable duration; nodes are then packed greedily, time test strict
 * (<), memory test <= per node, starting at the first_bubble-th fillable bubble and cycling.
 * out: host array of `cap` chunks (empty chunks are kept: chunk i belongs to fillable bubble
 * (first_bubble+i) mod n).  *n_out = chunk count (needed count on PF_ERR_CAPACITY);
 * *replicas = copies of F.  PF_ERR_INFEASIBLE when a node fits no bubble: *n_out then holds
 * the index in F of the first such node. */
int32_t pf_plan_bubbles(const pf_bubble* B, int32_t nB, const pf_node* F, int32_t nF,
                        int64_t fill_ppm, int64_t switch_ns, int32_t first_bubble,
                        pf_chunk* out, int32_t cap, int32_t* n_out, int32_t* replicas);

/* ---- Scheduler (Sec. 4.4) and event-driven simulation (Sec. 5.1) --------------------------------- */
enum { PF_POLICY_FIFO = 0, PF_POLICY_SJF = 1, PF_POLICY_MAKESPAN = 2 };
typedef struct pf_job { int64_t arrival_ns; int64_t deadline_ns; /* < 0: none (kept for callers; no policy here reads it) */ } pf_job;
typedef struct pf_job_run { int64_t start_ns, finish_ns; int32_t device, reserved; } pf_job_run;

/* Processing time of a fill job on a device (Sec. 4.4: computed from the job's profile, the
 * partitioning algorithm and the device's bubble description): the chain F is planned onto the
 * cycle `bubbles` by Algorithm 1 from bubble 0; one pass of the plan completes replicas *
 * samples_per_replica samples in ceil(chunks / fillable bubbles) cycles; the job needs
 * ceil(total_samples / that) passes; a cycle lasts iter_ns (one iteration of the main job).
 * *proc_ns (host, out) = passes * cycles * iter_ns.  Planner errors pass through
 * (PF_ERR_INFEASIBLE: the job does not fit this device). */
int32_t pf_job_time(const pf_bubble* bubbles, int32_t n_bubbles, const pf_node* F, int32_t nF,
                    int64_t samples_per_replica, int64_t total_samples, int64_t iter_ns, int64_t fill_ppm,
                    int64_t switch_ns, int64_t* proc_ns);

/* Event-driven simulation of n_jobs fill jobs on n_dev Executors.  proc_ns (host): [n_jobs][n_dev]
 * positive processing times.  Events are arrivals and completions; at an event every idle device, in
 * index order, is given the waiting job with the largest policy score f(j, s, i):
 *   PF_POLICY_FIFO      earliest arrival;
 *   PF_POLICY_SJF       1 / min(j.proc_times);
 *   PF_POLICY_MAKESPAN  1 / max(j.proc_times[i], max(s.rem_times)), rem_times = remaining busy time of
 *                       every Executor at that moment.
 * Ties: earlier arrival, then lower job index.  runs (host, out): device, start and finish per job.
 * makespan_ns / sum_completion_ns (host, out, may be NULL): latest finish; sum over jobs of finish -
 * arrival.  Jobs are not preempted and run whole on one device. */
int32_t pf_sched_simulate(int32_t policy, const pf_job* jobs, int32_t n_jobs, int32_t n_dev,
                          const int64_t* proc_ns, pf_job_run* runs, int64_t* makespan_ns,
                          int64_t* sum_completion_ns);

/* Bubble characterisation by the doubling probe (Sec. 4.2, "Bubble characterization"): how long
 * can stage `stage` of a p-stage, m-microbatch 1F1B pipeline (forward tf_ns, backward tb_ns per
 * microbatch and stage, no communication time) hold back at each of its bubble instructions before
 * the main job slows down.  The pipeline is simulated from its dependencies (forward j of a stage
 * needs forward j of the stage before, backward j the backward j of the stage after, a stage runs
 * its instructions in order).  The bubble instructions are taken one after the other in program
 * order, the waits already found staying in place: the wait starts at first_wait_ns and doubles
 * while the steady-state iteration period stays <= the undisturbed period * (1 + tol_ppm / 1e6);
 * the estimate is the last wait that passed (0 if first_wait_ns already slows the pipeline).  An
 * estimate can exceed the idle window it belongs to when a later window of the stage absorbs the
 * delay; the estimates together never slow the pipeline and sum to at most the stage's idle time.
 * est_ns (host, out): one value per idle window, same order and count as pf_schedule_1f1b.
 * PF_ERR_CAPACITY (count in *n_out) if cap is too small; PF_ERR_ARG on non-positive times. */
int32_t pf_probe_bubbles(int32_t p, int32_t m, int32_t stage, int64_t tf_ns, int64_t tb_ns,
                         int64_t first_wait_ns, int64_t tol_ppm, int64_t* est_ns, int32_t cap,
                         int32_t* n_out);

/* The same probe against the emulated stage (Sec. 4.2: the engine profiles at the start of the main job).  Stage
 * `stage` runs for real: its forward and backward instructions are executed by main_ctx on main_stream (as in
 * pf_main_stage_step, input / upstream gradient main_io) and their finish times are measured on the host; the
 * other p - 1 stages are simulated from tf_ns / tb_ns and from those measured times (forward j of a stage needs
 * forward j of the stage before, backward j the backward j of the stage after), and an instruction of the real
 * stage starts when the simulation says its input has arrived.  At bubble instruction k the stage holds back
 * for the trial wait.  A trial is four iterations; its period is the time between the ends of the last two.
 * The undisturbed period is the smaller of two trials without waits (*base_period_ns, may be NULL); the bubble
 * instructions are then probed one after the other exactly as in pf_probe_bubbles, with tol_ppm absorbing the
 * run-to-run noise of real kernels (1-2 % is typical).  est_ns, cap, n_out as in pf_probe_bubbles.
 * Synchronises main_stream after every instruction.  Takes about (4 * windows * log2(window / first_wait))
 * iterations of the stage.  PF_ERR_ARG if main_ctx has fewer checkpoint slots than min(p - stage, m). */
int32_t pf_probe_bubbles_live(pf_ctx* main_ctx, const void* main_io, int32_t p, int32_t m, int32_t stage,
                              int64_t tf_ns, int64_t tb_ns, int64_t first_wait_ns, int64_t tol_ppm,
                              int64_t* est_ns, int32_t cap, int32_t* n_out, int64_t* base_period_ns,
                              void* main_stream);

/* Plan of the main job's optimizer-state offload (Sec. 4.2, "Main job offloading"): the moment
 * estimates are only read by the optimizer update, so part of them leaves the device while the
 * iteration runs and the idle windows gain that memory.  One slice leaves with each of the m
 * forward instructions of stage `stage` (1F1B, p stages), on a stream of its own; everything comes
 * back during the gradient synchronisation of sync_ns that follows the stage's last backward.
 * A slice is the largest multiple of 256 bytes that d2h_bytes_per_s moves within tf_ns (its copy
 * is over when its forward is, so no bubble instruction waits for it); the total is the smallest
 * of state_bytes rounded down to 256, m slices, and what h2d_bytes_per_s moves within sync_ns
 * rounded down to 256 (the optimizer update does not wait either); the forwards take full slices
 * first to last until the total is used up.
 * slice_bytes (host, out, m values): bytes leaving with forward 0..m-1.
 * extra_free (host, out, one value per idle window, same order and count as pf_schedule_1f1b):
 * bytes that are off the device while that window is open = the slices of the forwards before it
 * in program order; 0 for the fill-drain window, which follows the optimizer update.  The caller
 * adds them to the windows' free_bytes.
 * PF_ERR_CAPACITY (count in *n_windows) if cap is too small; PF_ERR_ARG on a bad argument
 * (non-positive tf_ns, negative sizes or rates, state_bytes >= 2^62). */
int32_t pf_offload_plan(int32_t p, int32_t m, int32_t stage, int64_t tf_ns, int64_t sync_ns,
                        int64_t state_bytes, int64_t d2h_bytes_per_s, int64_t h2d_bytes_per_s,
                        int64_t* slice_bytes, int64_t* extra_free, int32_t cap, int32_t* n_windows);

/* Algorithm 1 for a job that arrives when its first bubble is partly gone (Sec. 4.3: the Executor
 * takes the next job as soon as one completes, which is in the middle of a bubble): exactly
 * pf_plan_bubbles, except that the FIRST visit of bubble `first_bubble` has the duration
 * first_dur_ns (what is left of it; the fill fraction and the switch time apply to it as to any
 * bubble) instead of its dur_ns.  Later visits of that bubble, and the replication count, use
 * dur_ns.  first_dur_ns < 0: no such shortening (identical to pf_plan_bubbles).  A first chunk
 * that takes no node is an ordinary empty chunk; being shortened, it does not count among the
 * consecutive empty chunks after which a node is declared to fit no bubble (PF_ERR_INFEASIBLE). */
int32_t pf_plan_bubbles_from(const pf_bubble* bubbles, int32_t n_bubbles, const pf_node* F, int32_t nF,
                             int64_t fill_ppm, int64_t switch_ns, int32_t first_bubble,
                             int64_t first_dur_ns, pf_chunk* out, int32_t cap, int32_t* n_out,
                             int32_t* replicas);

/* Configuration choice (Sec. 4.1/4.3: the plan that maximises throughput).  chains[c] (host) has
 * n_nodes[c] nodes and processes samples[c] samples per replica.  Every configuration is
 * planned as above; the winner maximises samples*replicas / ceil(chunks / fillable bubbles),
 * compared exactly in 128-bit integers; ties go to the smaller peak memory, then the lower
 * index.  Infeasible configurations are skipped.  *best = -1 with PF_ERR_INFEASIBLE when none
 * is feasible.  replicas_out / cycles_out / chunks_out (host, n_cfg entries each, may be NULL)
 * receive per-configuration results (0 for infeasible ones). */
int32_t pf_select_config(const pf_bubble* B, int32_t nB, const pf_node* const* chains,
                         const int32_t* n_nodes, const int64_t* samples, int32_t n_cfg,
                         int64_t fill_ppm, int64_t switch_ns, int32_t first_bubble,
                         int32_t* best, int32_t* replicas_out, int32_t* cycles_out,
                         int32_t* chunks_out);

/* Configuration choice for a stream of jobs of one kind (Sec. 4.3: when a fill job completes the Executor takes the
 * next one, which starts in what is left of the same bubble).  A plan of ONE job counts the rest of the bubble in
 * which the job ends as used up, which favours configurations whose single job happens to end near a bubble's
 * end.  Here configuration c is compared on a run of r_c = max(1, ceil(horizon_cycles * U / dur(F_c))) jobs back
 * to back, U = summed usable duration of the fillable bubbles of one cycle (fill fraction and switch time applied
 * as in pf_plan_bubbles): the run's chain is F_c repeated r_c times and processes samples[c] * r_c samples; the
 * runs are then compared exactly as in pf_select_config (same tie-breaks, infeasible ones skipped).
 * runs_out / cycles_out / chunks_out (host, n_cfg entries each, may be NULL): r_c, and the cycles and chunks the
 * run's plan takes (0 for infeasible configurations).  horizon_cycles >= 1. */
int32_t pf_select_config_stream(const pf_bubble* B, int32_t nB, const pf_node* const* chains,
                                const int32_t* n_nodes, const int64_t* samples, int32_t n_cfg,
                                int64_t fill_ppm, int64_t switch_ns, int32_t first_bubble,
                                int32_t horizon_cycles, int32_t* best, int32_t* runs_out, int32_t* cycles_out,
                                int32_t* chunks_out);

/* ---- job description -> chain of nodes (Sec. 4.3: the job's graph is flattened into a chain) ---- */
/* Writes the node list of one replica (g microbatches): [EMBED] L x LAYER_FWD FINAL_LN, and for
 * training HEAD_LOSS, L x LAYER_BWD (last layer first), OPT.  mem_bytes is the node's peak HBM
 * footprint including everything kept resident between bubbles; dur_ns is left 0 (fill it with
 * pf_profile_chain or by hand).  out: host, cap entries. */
int32_t pf_build_chain(const pf_model_desc* model, const pf_exec_config* cfg,
                       pf_node* out, int32_t cap, int32_t* n_out);

/* ---- packed layer weights -------------------------------------------------------------------
 * A layer blob holds, in model dtype, at 256-byte aligned offsets, in this order:
 *   0 ln1_g[d] 1 ln1_b[d] 2 w_qkv[3d][d] 3 b_qkv[3d] 4 w_o[d][d] 5 b_o[d]
 *   6 ln2_g[d] 7 ln2_b[d] 8 w_1[f][d] 9 b_1[f] 10 w_2[d][f] 11 b_2[d]
 * Matrices are [out_features][in_features], row-major (y = x W^T + b).  Rows 0..d-1 of w_qkv
 * produce Q, d..2d-1 K, 2d..3d-1 V; head i owns rows i*d_head..(i+1)*d_head of each block.
 * offsets: host array of 12 entries.  Returns the blob size in bytes (<0: error code). */
int64_t pf_layer_blob_layout(const pf_model_desc* model, int64_t* offsets);

/* ---- execution context --------------------------------------------------------------------- */
/* Bytes of arena pf_ctx_create needs for this model and configuration (<0: error code). */
int64_t pf_ctx_arena_bytes(const pf_model_desc* model, const pf_exec_config* cfg);
/* arena: device memory, 256-byte aligned, arena_bytes long, owned by the caller and kept alive
 * until pf_ctx_destroy.  PF_ERR_NOMEM if it is too small.  adam may be NULL for inference. */
int32_t pf_ctx_create(const pf_model_desc* model, const pf_exec_config* cfg, const pf_weights* w,
                      const pf_adam* adam, void* arena, int64_t arena_bytes, pf_ctx** out);
int32_t pf_ctx_destroy(pf_ctx* ctx);
/* Waits for all work the context has enqueued (fill, copy and main streams it has seen). */
int32_t pf_ctx_sync(pf_ctx* ctx);
/* Rings of job inputs and outputs (device).  Replica r of the chain reads input slot r mod n_in
 * (int32 token ids [g][batch][seq] when vocab > 0, else hidden states [g][batch][seq][d] in
 * model dtype) and writes its final hidden states [g][batch][seq][d] to output slot r mod n_out.
 * For training jobs `out` may be NULL. */
int32_t pf_ctx_set_io(pf_ctx* ctx, const void* in, int32_t n_in, void* out, int32_t n_out);

/* Host->HBM prefetch of one layer blob (Sec. 4.5: parameters offloaded to CPU memory).  Enqueues
 * on copy_stream: wait until the last kernels that read `slot` have finished, copy layer
 * `layer` from pinned host memory into the slot, record the slot's ready event.  A later
 * LAYER_FWD of that layer on the fill stream waits for the event.  copy_stream NULL = the
 * context's own copy stream (the one its automatic prefetch uses); with any other stream the copy
 * also waits for an earlier copy into the same slot that was enqueued elsewhere.  The chunk
 * runner finds the layer in the slot and does not copy it again; it goes on prefetching the
 * layers that follow into the slots after `slot`.  PF_ERR_STATE if the configuration is not
 * streamed, PF_ERR_ARG if layer or slot is out of range. */
int32_t pf_load_layer_async(pf_ctx* ctx, int32_t layer, int32_t slot, void* copy_stream);

/* Run one chunk's forward-type nodes (EMBED, LAYER_FWD, FINAL_LN, HEAD_LOSS) on fill_stream
 * (Sec. 4.3: the Executor runs the current partition in the current bubble).  F/nF: the chain the
 * plan was made from (host).  The hidden states cut by the end of the chunk stay in the
 * context until the next chunk (inter-bubble context).  act_in (device, may be NULL): overrides
 * the source of the chunk's first node (token ids for EMBED, else hidden states
 * [g][batch][seq][d]).  act_out (device, may be NULL): receives a copy of the hidden states
 * after the chunk's last node.  PF_ERR_NOMEM, before any launch, if chunk->mem_bytes exceeds
 * cap_bytes (the bubble's free memory; <= 0 disables the check); PF_ERR_STATE if the chunk holds
 * a backward-type node. */
int32_t pf_fill_chunk_fwd(pf_ctx* ctx, const pf_chunk* chunk, const pf_node* F, int32_t nF,
                          const void* act_in, void* act_out, int64_t cap_bytes, void* fill_stream);
/* Same for backward-type nodes (LAYER_BWD with recompute from the layer's checkpoint, OPT).
 * grad_io (device, may be NULL): overrides the upstream gradient [g][batch][seq][d] entering the
 * chunk's first node; after the call it is not modified.  grad_out (device, may be NULL)
 * receives a copy of the gradient leaving the chunk's last LAYER_BWD node. */
int32_t pf_fill_chunk_bwd(pf_ctx* ctx, const pf_chunk* chunk, const pf_node* F, int32_t nF,
                          const void* grad_io, void* grad_out, int64_t cap_bytes, void* fill_stream);
/* Convenience: run any chunk, dispatching each node to the forward or backward path. */
int32_t pf_fill_chunk(pf_ctx* ctx, const pf_chunk* chunk, const pf_node* F, int32_t nF,
                      int64_t cap_bytes, void* fill_stream);

/* Measure dur_ns of every node of F (host, in/out) on this device: each node is run `reps`
 * times after `warmup` runs on `stream` and the median HIP-event time is stored (the
 * per-node profiles the Executor is handed, Sec. 4.3).  Synchronises the device.
 * The nodes really run, on input slot 0 of the ring: call it between jobs, with no replica in
 * flight (carried hidden states, checkpoints and output slot 0 are overwritten).  On a training context the optimizer nodes run
 * the Adam kernel with a zero step (parameters, moment estimates, step count, accumulated loss and
 * gradient accumulators are the same after the call as before); PF_ERR_STATE if microbatches are
 * accumulated towards an optimizer step when it is called. */
int32_t pf_profile_chain(pf_ctx* ctx, pf_node* F, int32_t nF, int32_t warmup, int32_t reps,
                         void* stream);

/* Emulated main-job stage (Sec. 4.2).  ctx must be a training context with vocab == 0 whose
 * layers are the stage's layers.  PF_INSTR_FWD: forward of microbatch `index` through all
 * layers, keeping per-layer checkpoints; PF_INSTR_BWD: recompute + backward of microbatch
 * `index`, accumulating weight gradients.  `io`: device hidden states [batch][seq][d] (input
 * for FWD; upstream gradient for BWD).  PF_INSTR_OPT: Adam update of all the stage's parameters
 * from the gradients accumulated over `index` microbatches (index >= 1; io is ignored and may be
 * NULL), working copies recast, accumulators cleared.  Enqueues on main_stream and returns.
 * Microbatch `index` uses checkpoint slot index mod g of the context (g of its pf_exec_config), from
 * its forward to its backward: the context needs g >= the number of microbatches the schedule keeps
 * in flight on the stage (1F1B: min(p - stage, m)).  PF_ERR_STATE if a forward lands on a slot whose
 * backward has not run, or a backward on a slot without a forward.
 * PF_INSTR_BUBBLE is handled by pf_timeline_run and is rejected here with PF_ERR_ARG. */
int32_t pf_main_stage_step(pf_ctx* ctx, int32_t instr, int32_t index, const void* io,
                           void* main_stream);

/* What the stage hands to its neighbours (Sec. 4.2: the engine's send instructions follow the compute ones): copies
 * to dst (device, [batch][seq][d], model dtype) what = 0: the output of the forward of microbatch `index` (valid
 * from its forward until the slot's next forward), what = 1: the gradient with respect to the stage's input left
 * by the backward of microbatch `index` (valid until the slot's next backward).  Enqueues on stream.
 * PF_ERR_CAPACITY if dst_bytes is too small, PF_ERR_STATE if ctx is not a main-stage context. */
int32_t pf_main_stage_read(pf_ctx* ctx, int32_t what, int32_t index, void* dst, int64_t dst_bytes, void* stream);

/* Result of one emulated main-job iteration. */
typedef struct pf_timeline_stats {
  int64_t iter_ns;          /* wall time of the iteration                                        */
  int64_t offered_ns;       /* sum of the durations of the fillable bubbles visited              */
  int64_t idle_ns;          /* sum of all idle windows (fillable or not)                         */
  int64_t fill_busy_ns;     /* fill-stream busy time inside the bubbles (HIP events)             */
  int64_t overrun_ns;       /* fill work still running after its bubble's deadline, summed       */
  int64_t main_busy_ns;     /* main-stream busy time (0 when the main stage is a placeholder)    */
  int32_t chunks_run;       /* non-empty chunks executed                                         */
  int32_t replicas_done;    /* replicas of the chain completed in this iteration                 */
  int64_t offload_wait_ns;  /* host time the main stage was held up by its own offload copies:
                               at bubble instructions and before the optimizer update            */
  int64_t offloaded_bytes;  /* optimizer-state bytes that left the device and came back          */
} pf_timeline_stats;

/* Optimizer phase of the emulated main stage, and offload of its optimizer state around it
 * (Sec. 4.2, "Main job offloading" and step 2 of "Bubble signaling").
 * pf_main_opt_state_bytes: *bytes = size of the stage's Adam moment estimates (two fp32 values
 * per parameter), seen as one byte string: first and second moments of layer 0, of layer 1, ...
 * pf_ctx_set_main_offload, sync_ns >= 0: from now on pf_timeline_run with this main_ctx ends the
 * stage's work of an iteration, after its last backward and before the fill-drain window, with a
 * gradient synchronisation (no peers here: the main stream idles for sync_ns) followed by
 * PF_INSTR_OPT over the m microbatches.  sync_ns < 0 switches the phase off again (the default).
 * slice_bytes/n_slices (host; n_slices == 0: no offload, else n_slices must equal the m of the
 * timeline, e.g. from pf_offload_plan): with forward instruction j the next slice_bytes[j] bytes
 * of the string are copied to host_buf (pinned host memory the caller owns and keeps alive,
 * host_bytes >= the sum) on a stream of the context's own; every bubble instruction first waits
 * for the copies under way; the synchronisation starts the copies back and the optimizer update
 * waits for them.  Time the main stage loses to either wait is reported as offload_wait_ns.
 * scrub != 0: at each bubble instruction what has left the device is overwritten there with 0xff
 * bytes (as a fill job using that memory would), so a caller can check that the state comes back
 * intact.  Slices must be multiples of 4 bytes and sum to at most the state.
 * Errors: PF_ERR_ARG, PF_ERR_STATE (not a main-stage context), PF_ERR_CAPACITY (host_bytes). */
int32_t pf_main_opt_state_bytes(pf_ctx* main_ctx, int64_t* bytes);
int32_t pf_ctx_set_main_offload(pf_ctx* main_ctx, int64_t sync_ns, void* host_buf, int64_t host_bytes,
                                const int64_t* slice_bytes, int32_t n_slices, int32_t scrub);

/* What the Executor does when a plan completes (all its replicas ran) in the middle of a bubble
 * cycle.  enable == 0 (the default): the same plan is reused and the remaining windows of the
 * cycle stay empty until its first bubble comes round again.  enable != 0: the completed fill
 * job is followed at once by the next one (Sec. 4.3: the Executor asks for the next job when
 * one completes): the chain is partitioned again by Algorithm 1 with fill_ppm / switch_ns,
 * starting in the window that took the last chunk (pf_plan_bubbles_from with first_dur_ns =
 * the window's duration less ceil(planned duration of the chunks already launched in it * 1e6 /
 * fill_ppm), so the new job is charged its own switch time there); the new plan is kept
 * inside the context and replaces the caller's plan in later pf_timeline_run calls on it.  Every
 * call of this function drops a plan kept earlier (call it when the windows or the chain
 * change).  PF_ERR_ARG on a bad fraction or switch time. */
int32_t pf_ctx_set_replan(pf_ctx* ctx, int32_t enable, int64_t fill_ppm, int64_t switch_ns);

/* One iteration of an emulated 1F1B stage with the Executor's bubble loop inside it
 * (Sec. 4.2 signalling, Sec. 4.3 "Bubble synchronization and memory capping").
 * windows/nW: the stage's idle windows in time order (from pf_schedule_1f1b).  The stage's busy
 * periods between windows are real kernels when main_ctx != NULL (FWD/BWD of `main_io`,
 * issued in 1F1B order for p, m, stage; PF_ERR_ARG if main_ctx has fewer checkpoint slots, g, than the
 * min(p - stage, m) microbatches in flight) and timed waits of tf_ns / tb_ns otherwise.  At each fillable window the
 * next planned chunk plan[*cursor] whose bubble index equals the window is launched on
 * fill_stream with the window's free_bytes as cap, and the window is held open on the host for
 * its dur_ns.  fill_ctx may be NULL (no filling: the baseline for slowdown).  *cursor (host,
 * in/out) advances over plan[0..n_plan); when it reaches n_plan it wraps to 0 and the next
 * plan pass serves new replicas (same plan, or a new one: pf_ctx_set_replan; *cursor then
 * indexes the plan kept in the context).  Synchronises the device at the end.
 * Explicit cycles: with p == 0 (m, stage, tf_ns, tb_ns ignored, main_ctx must be NULL) the windows are
 * taken as given: before window k the fill and copy streams stay idle for start_ns[k] minus the end
 * of window k-1 (start_ns[0] for the first), then the window opens for dur_ns[k]. */
int32_t pf_timeline_run(pf_ctx* fill_ctx, pf_ctx* main_ctx, const void* main_io,
                        int32_t p, int32_t m, int32_t stage, int64_t tf_ns, int64_t tb_ns,
                        const pf_bubble* windows, int32_t nW,
                        const pf_chunk* plan, int32_t n_plan, const pf_node* F, int32_t nF,
                        int32_t* cursor, void* fill_stream, void* main_stream,
                        pf_timeline_stats* stats);

/* Scalar training state of a context: *loss = mean of the HEAD_LOSS values since the last call
 * (device sync), *steps = optimizer steps taken.  Either may be NULL. */
int32_t pf_ctx_train_state(pf_ctx* ctx, double* loss, int64_t* steps);

/* Copy parameter gradients / master weights of layer `layer` (blob layout, fp32 elements at the
 * same element order) to `dst` (device, fp32).  what: 0 accumulated gradients, 1 master weights,
 * 2 first-moment estimates, 3 second-moment estimates.
 * layer == -1: tok_emb | pos_emb | lnf_g | lnf_b concatenated.  For tests of training jobs. */
int32_t pf_ctx_read_params(pf_ctx* ctx, int32_t what, int32_t layer, void* dst, int64_t dst_bytes,
                           void* stream);

/* Sampling for pf_ctx_kernel_timing: only every n-th launch of an enabled class is bracketed by events
 * (n >= 1, default 1; PF_K_COPY_WAIT is never sampled).  An event pair costs about 10 us of stream time around the launch it brackets, so a
 * caller that times a kernel inside a throughput measurement samples it. */
int32_t pf_ctx_kernel_timing_every(pf_ctx* ctx, int32_t n);

/* Per-kernel-class timing.  mask: bit k enables class PF_K_k; enabled launches are bracketed by HIP
 * events on the stream they run on (a fixed pool of 16384 pairs between two reads; launches
 * beyond it run untimed).  pf_ctx_kernel_stats synchronises the device, folds the pool into the
 * totals and returns the class's launch count and summed duration since timing was enabled. */
int32_t pf_ctx_kernel_timing(pf_ctx* ctx, uint32_t mask);
int32_t pf_ctx_kernel_stats(pf_ctx* ctx, int32_t cls, int64_t* count, int64_t* total_ns);

/* ---- single kernels (the steps a layer visit is made of; used by tests and by the roofline
 * measurement).  All pointers device; `dtype` = storage type; fp32 accumulation throughout. ------ */
/* C[M,N] = X[M,K] * W[N,K]^T (+ bias[N]) (GELU if gelu) (+ resid[M,N]); C is fp32 if out_f32 (then
 * accumulate != 0 adds to C's old contents), else dtype.  bf16: K must be a multiple of 8.
 * The two forms the training backward uses (both may be NULL):
 * preact_out [M,N] (dtype): also receives X W^T + bias, the value before the GELU (kept for the backward pass);
 * dact_in [M,N] (dtype): the result is multiplied element-wise by GELU'(dact_in) (backward through the
 * activation: dU = (dY W_2) * GELU'(U)); not combined with bias, gelu, resid or preact_out. */
int32_t pf_op_gemm(int32_t dtype, const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K,
                   const void* bias, const void* resid, int32_t gelu, int32_t out_f32, int32_t accumulate,
                   const void* dact_in, void* preact_out, void* stream);
/* y = g * (x - mean) / sqrt(var + eps) + b per row; d a multiple of 8, at most 8192.
 * mean_out / rstd_out: fp32 [rows], may be NULL.
 * warm / warm_bytes (device, may be NULL / 0): the kernel also reads the whole 16-byte pieces inside
 * [warm, warm + warm_bytes) and discards them, which leaves them in the memory-side cache; the layer passes
 * the weights of the GEMMs that follow.  The range must be readable device memory; y does not depend on it. */
int32_t pf_op_layernorm(int32_t dtype, const void* x, const void* g, const void* b, void* y,
                        float* mean_out, float* rstd_out, int64_t rows, int32_t d, float eps, const void* warm,
                        int64_t warm_bytes, void* stream);
/* softmax(Q K^T / sqrt(dh) [+ causal mask]) V per (batch, head).  qkv: [B*S][3*h*dh] (Q | K | V
 * column blocks), out: [B*S][h*dh], lse: fp32 [B][h][S] or NULL.  dh in {8,16,32,64,128}. */
int32_t pf_op_attention(int32_t dtype, const void* qkv, void* out, float* lse, int32_t B, int32_t S,
                        int32_t h, int32_t dh, int32_t causal, void* stream);
/* Backward of pf_op_attention from the saved lse: dqkv [B*S][3*h*dh] receives dQ | dK | dV.  out / dout:
 * [B*S][h*dh]; dsum: fp32 scratch [B][h][S]. */
int32_t pf_op_attention_bwd(int32_t dtype, const void* qkv, const void* out, const void* dout, const float* lse,
                            float* dsum, void* dqkv, int32_t B, int32_t S, int32_t h, int32_t dh, int32_t causal,
                            void* stream);
/* Backward of pf_op_layernorm from the saved row statistics: dx = rstd * (g*dy - mean(g*dy) -
 * xhat * mean(g*dy*xhat)) (+ resid, same shape, may be NULL), dg += sum over rows of dy*xhat,
 * db += sum over rows of dy (dg, db: fp32 [d], accumulated into).  dx may alias resid or dy.
 * partial: fp32 scratch of 512 * 2 * d elements.  d a multiple of 8, at most 8192. */
int32_t pf_op_layernorm_bwd(int32_t dtype, const void* dy, const void* x, const void* g, const float* mean,
                            const float* rstd, const void* resid, void* dx, float* dg, float* db, float* partial,
                            int64_t rows, int32_t d, void* stream);
/* pf_op_layernorm_bwd for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without `partial`, same results.
 * The partial dg / db rows go to a device array of 8 MiB that the library holds on every GPU it runs on until the
 * process ends; its address on the current device is looked up on the first call there.  The call allocates
 * nothing.  d a multiple of 8, at most 8192 (PF_ERR_ARG beyond that); any number of rows (the array bounds the
 * number of workgroups, 128 at d = 8192, 512 up to d = 2048, not the input).  dx is identical to
 * pf_op_layernorm_bwd's; dg and db can differ in the last bits when rows exceeds the number of workgroups (fewer,
 * longer partial sums).  All calls on one GPU share the array: calls that overlap there (different streams or
 * threads) race; calls on one stream are safe. */
int32_t pf_op_layernorm_bwd_static(int32_t dtype, const void* dy, const void* x, const void* g, const float* mean,
                                   const float* rstd, const void* resid, void* dx, float* dg, float* db,
                                   int64_t rows, int32_t d, void* stream);
/* out[c][r] = in[r][c] for in [rows][cols], out [cols][rows] (distinct buffers); rows <= 64 * 65535.
 * colsum_acc (device fp32 [cols], may be NULL): colsum_acc[c] += sum over r of in[r][c] (fp32 atomics:
 * the order of the additions, and with it the last bits, can differ between calls). */
int32_t pf_op_transpose(int32_t dtype, const void* in, void* out, int64_t rows, int64_t cols, float* colsum_acc,
                        void* stream);
/* C[M][N] (device fp32, accumulated into) += A^T B for A [K][M] and B [K][N], row-major bf16: the weight
 * gradient dW = dY^T X of a linear layer from dY [tokens][n_out] and X [tokens][n_in] as they lie in memory.
 * colsum_acc (device fp32 [M], may be NULL): colsum_acc[m] += sum over k of A[k][m] (the bias gradient).
 * dtype must be PF_DTYPE_BF16, M and N multiples of 8, K a multiple of 64, A and B 16-byte aligned
 * (PF_ERR_ARG otherwise).  K may be split over workgroups that add into C with fp32 atomics: the last bits
 * of C and colsum_acc depend on the order of the additions. */
int32_t pf_op_gemm_tn(int32_t dtype, const void* A, const void* B, float* C, float* colsum_acc, int64_t M, int64_t N,
                      int64_t K, void* stream);
/* x[t] = tok[ids[t]] + pos[t mod S]; ids int32 [tokens]; ids outside [0,V) contribute zeros. */
int32_t pf_op_embed(int32_t dtype, const int32_t* ids, const void* tok, const void* pos, void* x,
                    int64_t tokens, int32_t S, int32_t d, int32_t V, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PIPEFILL_H */
