// Execution context of a fill job (internal).
#pragma once

#include <hip/hip_runtime.h>

#include <vector>

#include "pf_internal.h"

namespace pf {

// Sizes of everything a context keeps in HBM, derived from the model and the configuration.
// All regions are multiples of 256 bytes.
struct Layout {
  int32_t esz = 0;
  int64_t tokens = 0;        // per microbatch
  int64_t act = 0;           // one [tokens, d] tensor
  int64_t blob = 0;          // one packed layer
  int64_t off[12] = {};      // offsets inside a blob
  int64_t emb = 0;           // token + position embedding + final LayerNorm parameters
  // arena regions (bytes)
  int64_t slots = 0;         // streamed weight slots
  int64_t carried = 0;       // hidden states in flight (g microbatches)
  int64_t ws_fwd = 0;        // LN out, QKV, attention out, FFN mid
  int64_t total = 0;         // whole arena
  int64_t resident = 0;      // weights outside the arena that stay in HBM (resident layers, embeddings)
};

int32_t make_layout(const pf_model_desc& md, const pf_exec_config& cfg, Layout* out);

// Everything a training context (or the emulated main-job stage) keeps in its arena.
struct TrainState {
  int64_t Vp = 0;                       // vocabulary padded to a multiple of 64 (0: no embedding / head)
  int64_t blob32 = 0, off32[12] = {};   // fp32 layer layout (master weights, Adam moments, gradients)
  int64_t wt_off[4] = {}, wt_bytes = 0; // transposed w_qkv, w_o, w_1, w_2 inside a layer's transposed block
  int64_t emb32_off[4] = {}, emb32 = 0; // fp32 tok | pos | lnf_g | lnf_b
  std::vector<char*> Wk, Wt;            // working weights (model dtype, blob layout) and transposed matrices
  std::vector<float*> master, m, v, grad;
  char *E_w = nullptr, *Et = nullptr, *pos_w = nullptr, *lnf_g_w = nullptr, *lnf_b_w = nullptr;
  float *embM = nullptr, *embm = nullptr, *embv = nullptr, *embg = nullptr;
  char *ckpt = nullptr, *G = nullptr, *Hf = nullptr;
  char *ln2 = nullptr, *x1 = nullptr, *u = nullptr, *d_mid = nullptr, *d_qkv = nullptr, *d_attn = nullptr,
       *d_ln = nullptr, *tA = nullptr, *tB = nullptr, *logits = nullptr, *logitsT = nullptr;
  float *lse = nullptr, *Dsum = nullptr, *stats = nullptr, *ln_partial = nullptr, *loss = nullptr;
  int64_t stat_stride = 0;              // floats between the six per-token statistic arrays
  int64_t mb_accum = 0;                 // microbatches accumulated since the last optimizer step
  int64_t steps = 0;                    // optimizer steps taken
  int64_t loss_count = 0;               // HEAD_LOSS evaluations since the loss was last read
  bool dry = false;                     // profiling: optimizer steps leave parameters, moments and the step count alone
  std::vector<char> slot_live;          // emulated main stage: checkpoint slot holds a forward whose backward has not run
};

int64_t train_arena_bytes(const pf_model_desc& md, const pf_exec_config& cfg, const Layout& lay);

}  // namespace pf

struct pf_ctx;
namespace pf {
int32_t train_create(pf_ctx* c, const pf_weights* w, char* base, hipStream_t st);
void train_destroy(pf_ctx* c);
int32_t train_fwd_node(pf_ctx* c, const pf_node& n, int64_t replica, hipStream_t st);
int32_t train_bwd_node(pf_ctx* c, const pf_node& n, int64_t replica, const void* grad_in, hipStream_t st);
int32_t train_main_step(pf_ctx* c, int32_t instr, int32_t index, const void* io, hipStream_t st);
int32_t train_read_params(pf_ctx* c, int32_t what, int32_t layer, void* dst, int64_t dst_bytes, hipStream_t st);
// Optimizer state of a training context as one byte string: first and second moments of layer 0, of layer 1, ...
int64_t train_opt_state_bytes(const pf_ctx* c);
// copies bytes [off, off + len) of that string to (to_host) or from `host + off` (pinned host memory)
int32_t train_opt_state_copy(pf_ctx* c, int64_t off, int64_t len, char* host, bool to_host, hipStream_t st);
// overwrites bytes [off, off + len) of it with `byte`
int32_t train_opt_state_fill(pf_ctx* c, int64_t off, int64_t len, int32_t byte, hipStream_t st);
// optimizer update of an emulated main stage after `microbatches` accumulated backward passes
int32_t train_main_opt(pf_ctx* c, int32_t microbatches, hipStream_t st);
// Brackets pf_profile_chain on a training context: begin refuses a context with microbatches accumulated, saves the
// scalar state and switches optimizer steps to dry mode; end clears what the profiled nodes accumulated and restores it.
int32_t train_profile_begin(pf_ctx* c, hipStream_t st);
int32_t train_profile_end(pf_ctx* c, hipStream_t st);
// Weights that a LayerNorm reads ahead for the GEMMs after it: worth it while they are small beside the
// LayerNorm's own traffic and the cache they are meant to sit in; larger ranges are not warmed (returns 0).
inline int64_t warm_bytes(int64_t n) { return n <= ((int64_t)12 << 20) ? n : 0; }
// one pre-LN layer forward for one microbatch with the weights at wb (blob layout)
int32_t layer_forward(pf_ctx* c, const char* wb, const void* x_in, void* x_out, hipStream_t st);
}  // namespace pf

struct pf_ctx {
  pf_model_desc md{};
  pf_exec_config cfg{};
  pf_adam adam{};
  pf::Layout lay{};
  std::vector<void*> layers;      // device blobs (resident) or pinned host blobs (streamed)
  void* tok = nullptr;
  void* pos = nullptr;
  void* lnf_g = nullptr;
  void* lnf_b = nullptr;
  char* arena = nullptr;
  int64_t arena_bytes = 0;
  // arena regions
  char* slots = nullptr;
  char* X = nullptr;
  char* ws_ln = nullptr;
  char* ws_qkv = nullptr;
  char* ws_attn = nullptr;
  char* ws_mid = nullptr;
  // streamed-weights state
  std::vector<int32_t> slot_layer;
  std::vector<hipEvent_t> slot_ready, slot_free;
  std::vector<char> slot_free_valid;
  std::vector<hipStream_t> slot_stream;   // stream the slot's last copy was enqueued on
  int32_t next_slot = 0;
  hipStream_t copy_stream = nullptr;
  // job io rings
  const void* in = nullptr;
  int32_t n_in = 0;
  void* out = nullptr;
  int32_t n_out = 0;
  int64_t replica_base = 0;       // replicas completed by earlier passes over a cyclic plan
  bool replan = false;            // partition again, from the next bubble, when a plan completes
  int64_t replan_ppm = 1000000, replan_switch_ns = 0;
  std::vector<pf_chunk> active_plan;   // plan made by the last such re-partitioning (empty: caller's plan)
  // the hidden states currently carried come from here when the next node starts a replica
  int32_t device = 0;
  pf::TrainState* tr = nullptr;   // training contexts only
  // emulated main stage: optimizer phase after the last backward, and offload of the optimizer state around it
  struct MainOffload {
    bool opt_phase = false;          // gradient synchronisation (a wait of sync_ns) + optimizer update each iteration
    int64_t sync_ns = 0;
    char* host = nullptr;            // caller's pinned host buffer
    std::vector<int64_t> slices;     // bytes leaving with forward j (empty: nothing is offloaded)
    bool scrub = false;              // overwrite what has left the device until it comes back
    hipStream_t stream = nullptr;    // the copies' own stream
  } off;
  // optional per-kernel-class timing with HIP events on the launching stream
  struct TimedPair { hipEvent_t a, b; int32_t cls; };
  uint32_t timing_mask = 0;
  int32_t timing_every = 1;                      // bracket every n-th launch of an enabled class
  uint64_t cls_seen[PF_KERNEL_CLASSES] = {};
  std::vector<TimedPair> timing_pool;
  size_t timing_used = 0;
  int64_t cls_count[PF_KERNEL_CLASSES] = {};
  double cls_ms[PF_KERNEL_CLASSES] = {};
};
