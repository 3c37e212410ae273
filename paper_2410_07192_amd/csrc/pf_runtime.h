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
  int32_t next_slot = 0;
  hipStream_t copy_stream = nullptr;
  // job io rings
  const void* in = nullptr;
  int32_t n_in = 0;
  void* out = nullptr;
  int32_t n_out = 0;
  int64_t replica_base = 0;       // replicas completed by earlier passes over a cyclic plan
  // the hidden states currently carried come from here when the next node starts a replica
  int32_t device = 0;
  // optional per-kernel-class timing with HIP events on the launching stream
  struct TimedPair { hipEvent_t a, b; int32_t cls; };
  uint32_t timing_mask = 0;
  std::vector<TimedPair> timing_pool;
  size_t timing_used = 0;
  int64_t cls_count[PF_KERNEL_CLASSES] = {};
  double cls_ms[PF_KERNEL_CLASSES] = {};
};
