// Context, chunk runner, weight prefetch, node profiling and the emulated pipeline stage.
#include "pf_runtime.h"

#include <time.h>

#include <algorithm>
#include <cstring>
#include <new>

#include "pf_kernels.h"
#include "pf_pipeline_sim.h"

#define PF_HIP(expr)                                                                              \
  do {                                                                                            \
    hipError_t e__ = (expr);                                                                      \
    if (e__ != hipSuccess)                                                                        \
      return pf::fail(PF_ERR_HIP, "%s: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
  } while (0)

namespace pf {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

static bool bad_model(const pf_model_desc* m) {
  return !m || m->n_layers <= 0 || m->d_model <= 0 || m->n_heads <= 0 || m->d_ff <= 0 || m->seq_len <= 0 ||
         m->batch <= 0 || m->vocab < 0 || m->d_model % m->n_heads != 0 || m->d_model % 8 != 0 ||
         m->d_ff % 8 != 0 || (m->dtype != PF_DTYPE_F32 && m->dtype != PF_DTYPE_BF16) || !(m->eps >= 0.f);
}

static bool bad_cfg(const pf_exec_config* c) {
  return !c || c->g < 1 || (c->streamed && c->n_slots < 2) || c->n_slots < 0 || (c->training && c->streamed);
}

int32_t make_layout(const pf_model_desc& md, const pf_exec_config& cfg, Layout* L) {
  const int64_t e = esize(md.dtype), d = md.d_model, f = md.d_ff;
  L->esz = (int32_t)e;
  L->tokens = (int64_t)md.batch * md.seq_len;
  L->act = align_up(L->tokens * d * e, 256);
  const int64_t sizes[12] = {d, d, 3 * d * d, 3 * d, d * d, d, d, d, f * d, f, d * f, d};
  int64_t o = 0;
  for (int i = 0; i < 12; ++i) {
    L->off[i] = o;
    o += align_up(sizes[i] * e, 256);
  }
  L->blob = o;
  L->emb = md.vocab > 0 ? ((int64_t)md.vocab * d + (int64_t)md.seq_len * d) * e : 0;
  L->emb += 2 * d * e;
  L->slots = cfg.streamed ? (int64_t)cfg.n_slots * L->blob : 0;
  L->carried = (int64_t)cfg.g * L->act;
  L->ws_fwd = L->act /*LN out*/ + 3 * L->act /*QKV*/ + L->act /*attention out*/ +
              align_up(L->tokens * f * e, 256) /*FFN mid*/;
  L->total = L->slots + L->carried + L->ws_fwd;
  L->resident = L->emb + (cfg.streamed ? 0 : (int64_t)md.n_layers * L->blob);
  if (cfg.training) {
    // a training context copies every parameter into its arena and keeps checkpoints instead of one
    // carried tensor
    L->slots = 0;
    L->carried = 0;
    L->resident = 0;
    L->total = L->ws_fwd + train_arena_bytes(md, cfg, *L);
  }
  return PF_OK;
}

}  // namespace pf

using pf::Layout;

extern "C" {

const char* pf_last_error(void) { return pf::g_err; }
int32_t pf_version(void) { return 1; }

int64_t pf_layer_blob_layout(const pf_model_desc* model, int64_t* offsets) {
  if (pf::bad_model(model)) return pf::fail(PF_ERR_ARG, "pf_layer_blob_layout: bad model");
  Layout L;
  pf_exec_config c{1, 0, 0, 0};
  pf::make_layout(*model, c, &L);
  if (offsets) std::memcpy(offsets, L.off, sizeof L.off);
  return L.blob;
}

int64_t pf_ctx_arena_bytes(const pf_model_desc* model, const pf_exec_config* cfg) {
  if (pf::bad_model(model) || pf::bad_cfg(cfg)) return pf::fail(PF_ERR_ARG, "pf_ctx_arena_bytes: bad argument");
  Layout L;
  pf::make_layout(*model, *cfg, &L);
  return L.total;
}

int32_t pf_build_chain(const pf_model_desc* model, const pf_exec_config* cfg, pf_node* out, int32_t cap,
                       int32_t* n_out) {
  if (pf::bad_model(model) || pf::bad_cfg(cfg) || !n_out || cap < 0 || (cap > 0 && !out))
    return pf::fail(PF_ERR_ARG, "pf_build_chain: bad argument");
  if (cfg->training && model->vocab == 0)
    return pf::fail(PF_ERR_ARG, "pf_build_chain: a training fill job needs a vocabulary (embedding and tied head)");
  Layout L;
  pf::make_layout(*model, *cfg, &L);
  const int64_t persistent = L.resident + L.slots + L.carried;
  int32_t n = 0;
  auto put = [&](int32_t op, int32_t layer, int64_t mem) {
    if (n < cap) out[n] = pf_node{0, mem, op, layer, 0, cfg->g};
    ++n;
  };
  if (cfg->training) {
    // the whole arena (parameters, optimizer state, checkpoints, workspaces) stays allocated for the
    // life of the job, so every node reports it
    put(PF_OP_EMBED, -1, L.total);
    for (int32_t l = 0; l < model->n_layers; ++l) put(PF_OP_LAYER_FWD, l, L.total);
    put(PF_OP_FINAL_LN, -1, L.total);
    put(PF_OP_HEAD_LOSS, -1, L.total);
    for (int32_t l = model->n_layers - 1; l >= 0; --l) put(PF_OP_LAYER_BWD, l, L.total);
    put(PF_OP_OPT, -1, L.total);
    *n_out = n;
    if (n > cap) return pf::fail(PF_ERR_CAPACITY, "pf_build_chain: %d nodes, capacity %d", n, cap);
    return PF_OK;
  }
  if (model->vocab > 0) put(PF_OP_EMBED, -1, persistent);
  for (int32_t l = 0; l < model->n_layers; ++l) put(PF_OP_LAYER_FWD, l, persistent + L.ws_fwd);
  put(PF_OP_FINAL_LN, -1, persistent);
  *n_out = n;
  if (n > cap) return pf::fail(PF_ERR_CAPACITY, "pf_build_chain: %d nodes, capacity %d", n, cap);
  return PF_OK;
}

int32_t pf_ctx_create(const pf_model_desc* model, const pf_exec_config* cfg, const pf_weights* w,
                      const pf_adam* adam, void* arena, int64_t arena_bytes, pf_ctx** out) {
  if (pf::bad_model(model) || pf::bad_cfg(cfg) || !w || !w->layers || !arena || arena_bytes <= 0 || !out)
    return pf::fail(PF_ERR_ARG, "pf_ctx_create: bad argument");
  if (((uintptr_t)arena & 255) != 0) return pf::fail(PF_ERR_ARG, "pf_ctx_create: arena must be 256-byte aligned");
  if (cfg->training && adam && (adam->accum < 1 || !(adam->lr >= 0.f)))
    return pf::fail(PF_ERR_ARG, "pf_ctx_create: bad Adam constants");
  if (((!cfg->training || model->vocab > 0) && (!w->lnf_g || !w->lnf_b)) ||
      (model->vocab > 0 && (!w->tok_emb || !w->pos_emb)))
    return pf::fail(PF_ERR_ARG, "pf_ctx_create: missing embedding / final LayerNorm pointers");
  for (int32_t l = 0; l < model->n_layers; ++l)
    if (!w->layers[l]) return pf::fail(PF_ERR_ARG, "pf_ctx_create: layer %d pointer is null", l);
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0)
    return pf::fail(PF_ERR_HIP, "pf_ctx_create: no HIP device available (this library has no CPU path)");
  pf_ctx* c = new (std::nothrow) pf_ctx();
  if (!c) return pf::fail(PF_ERR_NOMEM, "pf_ctx_create: host allocation failed");
  c->md = *model;
  c->cfg = *cfg;
  c->adam = adam ? *adam : pf_adam{1e-4f, 0.9f, 0.999f, 1e-8f, 4};
  pf::make_layout(*model, *cfg, &c->lay);
  if (arena_bytes < c->lay.total) {
    const long long need = (long long)c->lay.total;
    delete c;
    return pf::fail(PF_ERR_NOMEM, "pf_ctx_create: arena has %lld bytes, %lld needed", (long long)arena_bytes, need);
  }
  c->layers.assign(w->layers, w->layers + model->n_layers);
  c->tok = w->tok_emb;
  c->pos = w->pos_emb;
  c->lnf_g = w->lnf_g;
  c->lnf_b = w->lnf_b;
  c->arena = (char*)arena;
  c->arena_bytes = arena_bytes;
  char* p = c->arena;
  c->slots = p; p += c->lay.slots;
  c->X = p; p += c->lay.carried;
  c->ws_ln = p; p += c->lay.act;
  c->ws_qkv = p; p += 3 * c->lay.act;
  c->ws_attn = p; p += c->lay.act;
  c->ws_mid = p; p += c->lay.ws_fwd - 5 * c->lay.act;
  hipError_t e = hipGetDevice(&c->device);
  if (e == hipSuccess && cfg->training) {
    int32_t rc = pf::train_create(c, w, p, nullptr);
    if (rc != PF_OK) {
      pf_ctx_destroy(c);
      return rc;
    }
  }
  if (e == hipSuccess && cfg->streamed) {
    c->slot_layer.assign(cfg->n_slots, -1);
    c->slot_free_valid.assign(cfg->n_slots, 0);
    c->slot_stream.assign(cfg->n_slots, nullptr);
    c->slot_ready.resize(cfg->n_slots);
    c->slot_free.resize(cfg->n_slots);
    for (int32_t i = 0; i < cfg->n_slots && e == hipSuccess; ++i) {
      e = hipEventCreateWithFlags(&c->slot_ready[i], hipEventDisableTiming);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&c->slot_free[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking);
  }
  if (e != hipSuccess) {
    pf_ctx_destroy(c);
    return pf::fail(PF_ERR_HIP, "pf_ctx_create: %s", hipGetErrorString(e));
  }
  *out = c;
  return PF_OK;
}

int32_t pf_ctx_destroy(pf_ctx* c) {
  if (!c) return PF_OK;
  (void)hipDeviceSynchronize();
  for (hipEvent_t ev : c->slot_ready) if (ev) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : c->slot_free) if (ev) (void)hipEventDestroy(ev);
  if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
  if (c->off.stream) (void)hipStreamDestroy(c->off.stream);
  if (c->tr) pf::train_destroy(c);
  for (auto& p : c->timing_pool) {
    if (p.a) (void)hipEventDestroy(p.a);
    if (p.b) (void)hipEventDestroy(p.b);
  }
  delete c;
  return PF_OK;
}

int32_t pf_ctx_sync(pf_ctx* c) {
  if (!c) return pf::fail(PF_ERR_ARG, "pf_ctx_sync: null context");
  PF_HIP(hipDeviceSynchronize());
  return PF_OK;
}

int32_t pf_ctx_set_io(pf_ctx* c, const void* in, int32_t n_in, void* out, int32_t n_out) {
  if (!c || n_in < 0 || n_out < 0 || (n_in > 0 && !in) || (n_out > 0 && !out))
    return pf::fail(PF_ERR_ARG, "pf_ctx_set_io: bad argument");
  c->in = in;
  c->n_in = n_in;
  c->out = out;
  c->n_out = n_out;
  return PF_OK;
}

// ---- weight streaming ---------------------------------------------------------------------------
static int32_t load_into(pf_ctx* c, int32_t layer, int32_t slot, hipStream_t cs) {
  if (c->slot_free_valid[slot]) PF_HIP(hipStreamWaitEvent(cs, c->slot_free[slot], 0));
  // an earlier copy into this slot that was enqueued on another stream must have landed first
  if (c->slot_layer[slot] >= 0 && c->slot_stream[slot] != cs) PF_HIP(hipStreamWaitEvent(cs, c->slot_ready[slot], 0));
  PF_HIP(hipMemcpyAsync(c->slots + (int64_t)slot * c->lay.blob, c->layers[layer], (size_t)c->lay.blob,
                        hipMemcpyHostToDevice, cs));
  PF_HIP(hipEventRecord(c->slot_ready[slot], cs));
  c->slot_layer[slot] = layer;
  c->slot_stream[slot] = cs;
  return PF_OK;
}

int32_t pf_load_layer_async(pf_ctx* c, int32_t layer, int32_t slot, void* copy_stream) {
  if (!c) return pf::fail(PF_ERR_ARG, "pf_load_layer_async: null context");
  if (!c->cfg.streamed) return pf::fail(PF_ERR_STATE, "pf_load_layer_async: configuration keeps weights resident");
  if (layer < 0 || layer >= c->md.n_layers || slot < 0 || slot >= c->cfg.n_slots)
    return pf::fail(PF_ERR_ARG, "pf_load_layer_async: layer %d / slot %d out of range", layer, slot);
  int32_t rc = load_into(c, layer, slot, copy_stream ? (hipStream_t)copy_stream : c->copy_stream);
  if (rc == PF_OK) c->next_slot = (slot + 1) % c->cfg.n_slots;
  return rc;
}

// ---- optional event timing of kernel classes ---------------------------------------------------------
struct TimedScope {
  pf_ctx* c;
  hipStream_t st;
  hipEvent_t end = nullptr;
  TimedScope(pf_ctx* ctx, int32_t cls, hipStream_t s) : c(ctx), st(s) {
    if (!((c->timing_mask >> cls) & 1u) || c->timing_used >= c->timing_pool.size()) return;
    if (cls != PF_K_COPY_WAIT && c->timing_every > 1 && (c->cls_seen[cls]++ % c->timing_every) != 0) return;   // sampled launches only (waits are summed: all of them count)
    pf_ctx::TimedPair& p = c->timing_pool[c->timing_used];
    if (hipEventRecord(p.a, st) != hipSuccess) return;
    p.cls = cls;
    end = p.b;
    ++c->timing_used;
  }
  ~TimedScope() {
    if (end) (void)hipEventRecord(end, st);
  }
};

static int32_t find_slot(const pf_ctx* c, int32_t layer) {
  for (int32_t i = 0; i < (int32_t)c->slot_layer.size(); ++i)
    if (c->slot_layer[i] == layer) return i;
  return -1;
}

// Makes `layer` available in a slot (loading it if no slot holds it), prefetches the layers that
// follow it into the other slots, and makes `fs` wait for the layer's copy.  Returns the slot.
static int32_t acquire_layer(pf_ctx* c, int32_t layer, hipStream_t fs, int32_t* slot_out) {
  const int32_t ns = c->cfg.n_slots, L = c->md.n_layers;
  int32_t s = find_slot(c, layer);
  if (s < 0) {
    s = c->next_slot;
    c->next_slot = (s + 1) % ns;
    int32_t rc = load_into(c, layer, s, c->copy_stream);
    if (rc != PF_OK) return rc;
  }
  for (int32_t t = 1; t < ns && t < L; ++t) {
    const int32_t nl = (layer + t) % L;
    if (find_slot(c, nl) >= 0) continue;
    int32_t ps = c->next_slot;
    if (ps == s) ps = (ps + 1) % ns;
    c->next_slot = (ps + 1) % ns;
    int32_t rc = load_into(c, nl, ps, c->copy_stream);
    if (rc != PF_OK) return rc;
  }
  {
    TimedScope t(c, PF_K_COPY_WAIT, fs);   // when enabled: how long the fill stream has nothing to run until the copy lands
    PF_HIP(hipStreamWaitEvent(fs, c->slot_ready[s], 0));
  }
  *slot_out = s;
  return PF_OK;
}

static int32_t drain_timing(pf_ctx* c) {
  PF_HIP(hipDeviceSynchronize());
  for (size_t i = 0; i < c->timing_used; ++i) {
    float ms = 0.f;
    const pf_ctx::TimedPair& p = c->timing_pool[i];
    if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
      c->cls_count[p.cls] += 1;
      c->cls_ms[p.cls] += ms;
    }
  }
  c->timing_used = 0;
  return PF_OK;
}

// ---- one layer, one microbatch -------------------------------------------------------------------
}  // extern "C"

int32_t pf::layer_forward(pf_ctx* c, const char* wb, const void* x_in, void* x_out, hipStream_t st) {
  const pf_model_desc& m = c->md;
  const int64_t* o = c->lay.off;
  const int64_t T = c->lay.tokens;
  const int32_t d = m.d_model, f = m.d_ff, dt = m.dtype;
  {
    TimedScope t(c, PF_K_LAYERNORM, st);
    PF_HIP(pf::layernorm_fwd(dt, x_in, wb + o[0], wb + o[1], c->ws_ln, nullptr, nullptr, T, d, m.eps, st, wb + o[2],
                             pf::warm_bytes(o[4] - o[2])));   // also warms W_qkv, b_qkv
  }
  pf::GemmEpilogue e1;
  e1.bias = wb + o[3];
  {
    TimedScope t(c, PF_K_GEMM_QKV, st);
    PF_HIP(pf::gemm_nt(dt, c->ws_ln, wb + o[2], c->ws_qkv, T, 3 * d, d, e1, st));
  }
  {
    TimedScope t(c, PF_K_ATTENTION, st);
    PF_HIP(pf::attention_fwd(dt, c->ws_qkv, c->ws_attn, nullptr, m.batch, m.seq_len, m.n_heads, d / m.n_heads,
                             m.causal, st));
  }
  pf::GemmEpilogue e2;
  e2.bias = wb + o[5];
  e2.resid = x_in;
  {
    TimedScope t(c, PF_K_GEMM_OUT, st);
    PF_HIP(pf::gemm_nt(dt, c->ws_attn, wb + o[4], x_out, T, d, d, e2, st));
  }
  {
    TimedScope t(c, PF_K_LAYERNORM, st);
    PF_HIP(pf::layernorm_fwd(dt, x_out, wb + o[6], wb + o[7], c->ws_ln, nullptr, nullptr, T, d, m.eps, st, wb + o[8],
                             pf::warm_bytes(c->lay.blob - o[8]) ? c->lay.blob - o[8] : pf::warm_bytes(o[10] - o[8])));   // W_1 .. b_2, or W_1 alone
  }
  pf::GemmEpilogue e3;
  e3.bias = wb + o[9];
  e3.gelu = 1;
  {
    TimedScope t(c, PF_K_GEMM_FFN1, st);
    PF_HIP(pf::gemm_nt(dt, c->ws_ln, wb + o[8], c->ws_mid, T, f, d, e3, st));
  }
  pf::GemmEpilogue e4;
  e4.bias = wb + o[11];
  e4.resid = x_out;
  {
    TimedScope t(c, PF_K_GEMM_FFN2, st);
    PF_HIP(pf::gemm_nt(dt, c->ws_mid, wb + o[10], x_out, T, d, f, e4, st));
  }
  return PF_OK;
}

extern "C" {

static int32_t check_chunk(const pf_ctx* c, const pf_chunk* ch, const pf_node* F, int32_t nF, int64_t cap,
                           const char* who) {
  if (!c || !ch || !F || nF <= 0) return pf::fail(PF_ERR_ARG, "%s: null argument", who);
  if (ch->node_begin < 0 || ch->node_end < ch->node_begin) return pf::fail(PF_ERR_ARG, "%s: bad node range", who);
  if (cap > 0 && ch->mem_bytes > cap)
    return pf::fail(PF_ERR_NOMEM, "%s: chunk needs %lld bytes, the bubble offers %lld", who,
                    (long long)ch->mem_bytes, (long long)cap);
  for (int32_t j = ch->node_begin; j < ch->node_end; ++j) {
    const pf_node& n = F[j % nF];
    if (n.mb_count != c->cfg.g)
      return pf::fail(PF_ERR_ARG, "%s: node %d visits %d microbatches, the context was made for %d", who, j % nF,
                      n.mb_count, c->cfg.g);
    if ((n.op == PF_OP_LAYER_FWD || n.op == PF_OP_LAYER_BWD) && (n.layer < 0 || n.layer >= c->md.n_layers))
      return pf::fail(PF_ERR_ARG, "%s: node %d names layer %d", who, j % nF, n.layer);
    if (n.op < PF_OP_EMBED || n.op > PF_OP_OPT) return pf::fail(PF_ERR_ARG, "%s: node %d has unknown op", who, j % nF);
    if (n.op == PF_OP_EMBED && c->md.vocab == 0)
      return pf::fail(PF_ERR_ARG, "%s: EMBED node but the model has no vocabulary", who);
  }
  return PF_OK;
}

int32_t pf_fill_chunk_fwd(pf_ctx* c, const pf_chunk* ch, const pf_node* F, int32_t nF, const void* act_in,
                          void* act_out, int64_t cap_bytes, void* fill_stream) {
  int32_t rc = check_chunk(c, ch, F, nF, cap_bytes, "pf_fill_chunk_fwd");
  if (rc != PF_OK) return rc;
  for (int32_t j = ch->node_begin; j < ch->node_end; ++j)
    if (F[j % nF].op > PF_OP_HEAD_LOSS)
      return pf::fail(PF_ERR_STATE, "pf_fill_chunk_fwd: node %d is a backward-type node", j % nF);
  hipStream_t st = (hipStream_t)fill_stream;
  const pf_model_desc& m = c->md;
  const int32_t g = c->cfg.g;
  const int64_t act = c->lay.act, T = c->lay.tokens;
  if (c->tr) {
    if (act_in || act_out)
      return pf::fail(PF_ERR_ARG, "pf_fill_chunk_fwd: act_in / act_out are not supported for training contexts");
    for (int32_t j = ch->node_begin; j < ch->node_end; ++j) {
      rc = pf::train_fwd_node(c, F[j % nF], c->replica_base + j / nF, st);
      if (rc != PF_OK) return rc;
    }
    return PF_OK;
  }
  const void* last_out = c->X;
  for (int32_t j = ch->node_begin; j < ch->node_end; ++j) {
    const pf_node& n = F[j % nF];
    const int64_t r = c->replica_base + j / nF;
    const bool first_of_chunk = (j == ch->node_begin);
    const bool starts_replica = (j % nF == 0);
    // where this node's input comes from
    const char* src = c->X;
    if (first_of_chunk && act_in) {
      src = (const char*)act_in;
    } else if (starts_replica) {
      if (!c->in || c->n_in <= 0) return pf::fail(PF_ERR_STATE, "pf_fill_chunk_fwd: no input ring set (pf_ctx_set_io)");
      const int64_t slot_bytes = (m.vocab > 0) ? (int64_t)g * T * 4 : (int64_t)g * act;
      src = (const char*)c->in + (r % c->n_in) * slot_bytes;
    }
    switch (n.op) {
      case PF_OP_EMBED:
        for (int32_t mb = 0; mb < g; ++mb)
          PF_HIP(pf::embed_fwd(m.dtype, (const int32_t*)src + mb * T, c->tok, c->pos, c->X + mb * act, T, m.seq_len,
                               m.d_model, m.vocab, st));
        last_out = c->X;
        break;
      case PF_OP_LAYER_FWD: {
        const char* wb;
        int32_t slot = -1;
        if (c->cfg.streamed) {
          rc = acquire_layer(c, n.layer, st, &slot);
          if (rc != PF_OK) return rc;
          wb = c->slots + (int64_t)slot * c->lay.blob;
        } else {
          wb = (const char*)c->layers[n.layer];
        }
        for (int32_t mb = 0; mb < g; ++mb) {
          rc = pf::layer_forward(c, wb, src + mb * act, c->X + mb * act, st);
          if (rc != PF_OK) return rc;
        }
        if (slot >= 0) {
          PF_HIP(hipEventRecord(c->slot_free[slot], st));
          c->slot_free_valid[slot] = 1;
        }
        last_out = c->X;
        break;
      }
      case PF_OP_FINAL_LN: {
        char* dst = c->X;
        if (c->out && c->n_out > 0) dst = (char*)c->out + (r % c->n_out) * ((int64_t)g * act);
        for (int32_t mb = 0; mb < g; ++mb)
          PF_HIP(pf::layernorm_fwd(m.dtype, src + mb * act, c->lnf_g, c->lnf_b, dst + mb * act, nullptr, nullptr, T,
                                   m.d_model, m.eps, st));
        last_out = dst;
        break;
      }
      default:
        return pf::fail(PF_ERR_STATE, "pf_fill_chunk_fwd: op %d is not available in this build", n.op);
    }
  }
  if (act_out && ch->node_end > ch->node_begin)
    PF_HIP(hipMemcpyAsync(act_out, last_out, (size_t)((int64_t)g * act), hipMemcpyDeviceToDevice, st));
  return PF_OK;
}

int32_t pf_fill_chunk_bwd(pf_ctx* c, const pf_chunk* ch, const pf_node* F, int32_t nF, const void* grad_io,
                          void* grad_out, int64_t cap_bytes, void* fill_stream) {
  int32_t rc = check_chunk(c, ch, F, nF, cap_bytes, "pf_fill_chunk_bwd");
  if (rc != PF_OK) return rc;
  if (!c->tr) return pf::fail(PF_ERR_STATE, "pf_fill_chunk_bwd: not a training context");
  for (int32_t j = ch->node_begin; j < ch->node_end; ++j)
    if (F[j % nF].op <= PF_OP_HEAD_LOSS)
      return pf::fail(PF_ERR_STATE, "pf_fill_chunk_bwd: node %d is a forward-type node", j % nF);
  hipStream_t st = (hipStream_t)fill_stream;
  bool saw_layer = false;
  for (int32_t j = ch->node_begin; j < ch->node_end; ++j) {
    const pf_node& n = F[j % nF];
    const void* gin = (j == ch->node_begin && n.op == PF_OP_LAYER_BWD) ? grad_io : nullptr;
    rc = pf::train_bwd_node(c, n, c->replica_base + j / nF, gin, st);
    if (rc != PF_OK) return rc;
    saw_layer = saw_layer || n.op == PF_OP_LAYER_BWD;
  }
  if (grad_out && saw_layer)
    PF_HIP(hipMemcpyAsync(grad_out, c->tr->G, (size_t)((int64_t)c->cfg.g * c->lay.act), hipMemcpyDeviceToDevice, st));
  return PF_OK;
}

int32_t pf_fill_chunk(pf_ctx* c, const pf_chunk* ch, const pf_node* F, int32_t nF, int64_t cap_bytes,
                      void* fill_stream) {
  int32_t rc = check_chunk(c, ch, F, nF, cap_bytes, "pf_fill_chunk");
  if (rc != PF_OK) return rc;
  // split the chunk into maximal runs of forward-type and backward-type nodes
  int32_t j = ch->node_begin;
  while (j < ch->node_end) {
    const bool bwd = F[j % nF].op > PF_OP_HEAD_LOSS;
    int32_t e = j;
    while (e < ch->node_end && (F[e % nF].op > PF_OP_HEAD_LOSS) == bwd) ++e;
    pf_chunk part = *ch;
    part.node_begin = j;
    part.node_end = e;
    rc = bwd ? pf_fill_chunk_bwd(c, &part, F, nF, nullptr, nullptr, 0, fill_stream)
             : pf_fill_chunk_fwd(c, &part, F, nF, nullptr, nullptr, 0, fill_stream);
    if (rc != PF_OK) return rc;
    j = e;
  }
  return PF_OK;
}

// ---- profiling -----------------------------------------------------------------------------------
int32_t pf_profile_chain(pf_ctx* c, pf_node* F, int32_t nF, int32_t warmup, int32_t reps, void* stream) {
  if (!c || !F || nF <= 0 || warmup < 0 || reps <= 0) return pf::fail(PF_ERR_ARG, "pf_profile_chain: bad argument");
  hipStream_t st = (hipStream_t)stream;
  if (c->tr) {
    int32_t brc = pf::train_profile_begin(c, st);
    if (brc != PF_OK) return brc;
  }
  std::vector<hipEvent_t> ev(nF + 1, nullptr);
  int32_t rc = PF_OK;
  for (auto& e : ev)
    if (rc == PF_OK && hipEventCreate(&e) != hipSuccess) rc = pf::fail(PF_ERR_HIP, "pf_profile_chain: hipEventCreate failed");
  std::vector<std::vector<float>> ms(nF);
  const int64_t saved_base = c->replica_base;
  for (int32_t it = 0; it < warmup + reps && rc == PF_OK; ++it) {
    // the whole chain runs in order so that streamed configurations are measured with their
    // copies overlapping the previous layer, as they do inside a bubble
    hipError_t he = hipEventRecord(ev[0], st);
    for (int32_t i = 0; i < nF && rc == PF_OK && he == hipSuccess; ++i) {
      pf_chunk one{0, 0, i, i + 1, 0, 0};
      rc = pf_fill_chunk(c, &one, F, nF, 0, st);
      if (rc == PF_OK) he = hipEventRecord(ev[i + 1], st);
    }
    if (rc == PF_OK && he == hipSuccess) he = hipStreamSynchronize(st);
    if (rc == PF_OK && he != hipSuccess) rc = pf::fail(PF_ERR_HIP, "pf_profile_chain: %s", hipGetErrorString(he));
    if (rc == PF_OK && it >= warmup)
      for (int32_t i = 0; i < nF; ++i) {
        float t = 0.f;
        he = hipEventElapsedTime(&t, ev[i], ev[i + 1]);
        if (he != hipSuccess) { rc = pf::fail(PF_ERR_HIP, "pf_profile_chain: %s", hipGetErrorString(he)); break; }
        ms[i].push_back(t);
      }
  }
  c->replica_base = saved_base;
  for (auto& e : ev) if (e) (void)hipEventDestroy(e);
  if (c->tr) {
    const int32_t erc = pf::train_profile_end(c, st);
    if (rc == PF_OK) rc = erc;
  }
  if (rc != PF_OK) return rc;
  for (int32_t i = 0; i < nF; ++i) {
    std::sort(ms[i].begin(), ms[i].end());
    const double med = ms[i][ms[i].size() / 2];
    F[i].dur_ns = (int64_t)(med * 1e6 + 0.5);
    if (F[i].dur_ns < 1) F[i].dur_ns = 1;
  }
  return PF_OK;
}

// ---- emulated pipeline stage -----------------------------------------------------------------------
static int64_t now_ns() {
  timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (int64_t)ts.tv_sec * 1000000000LL + ts.tv_nsec;
}

// sleep coarsely, then spin the last 150 us, until the monotonic clock reaches `deadline`
static void wait_until(int64_t deadline) {
  for (;;) {
    const int64_t left = deadline - now_ns();
    if (left <= 0) return;
    if (left > 200000) {
      timespec ts{0, (long)std::min<int64_t>(left - 150000, 2000000)};
      nanosleep(&ts, nullptr);
    }
  }
}

int32_t pf_main_stage_step(pf_ctx* c, int32_t instr, int32_t index, const void* io, void* main_stream) {
  if (!c || index < 0 || (!io && instr != PF_INSTR_OPT)) return pf::fail(PF_ERR_ARG, "pf_main_stage_step: bad argument");
  if (instr == PF_INSTR_BUBBLE)
    return pf::fail(PF_ERR_ARG, "pf_main_stage_step: the bubble instruction is executed by pf_timeline_run");
  if (instr != PF_INSTR_FWD && instr != PF_INSTR_BWD && instr != PF_INSTR_OPT)
    return pf::fail(PF_ERR_ARG, "pf_main_stage_step: unknown instruction");
  if (!c->tr || c->md.vocab != 0)
    return pf::fail(PF_ERR_STATE, "pf_main_stage_step: needs a training context without vocabulary");
  if (instr == PF_INSTR_OPT) {
    if (index < 1) return pf::fail(PF_ERR_ARG, "pf_main_stage_step: the optimizer update needs the number of microbatches");
    return pf::train_main_opt(c, index, (hipStream_t)main_stream);
  }
  return pf::train_main_step(c, instr, index, io, (hipStream_t)main_stream);
}

int32_t pf_main_stage_read(pf_ctx* c, int32_t what, int32_t index, void* dst, int64_t dst_bytes, void* stream) {
  if (!c || !dst || index < 0 || (what != 0 && what != 1)) return pf::fail(PF_ERR_ARG, "pf_main_stage_read: bad argument");
  if (!c->tr || c->md.vocab != 0)
    return pf::fail(PF_ERR_STATE, "pf_main_stage_read: needs a training context without vocabulary");
  if (dst_bytes < c->lay.act) return pf::fail(PF_ERR_CAPACITY, "pf_main_stage_read: %lld bytes needed", (long long)c->lay.act);
  const int64_t slot = index % c->cfg.g, L = c->md.n_layers;
  const char* src = what == 0 ? c->tr->ckpt + (slot * (L + 1) + L) * c->lay.act : c->tr->G + slot * c->lay.act;
  PF_HIP(hipMemcpyAsync(dst, src, (size_t)c->lay.act, hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return PF_OK;
}

int32_t pf_main_opt_state_bytes(pf_ctx* c, int64_t* bytes) {
  if (!c || !bytes) return pf::fail(PF_ERR_ARG, "pf_main_opt_state_bytes: bad argument");
  if (!c->tr || c->md.vocab != 0)
    return pf::fail(PF_ERR_STATE, "pf_main_opt_state_bytes: needs a training context without vocabulary");
  *bytes = pf::train_opt_state_bytes(c);
  return PF_OK;
}

int32_t pf_ctx_set_main_offload(pf_ctx* c, int64_t sync_ns, void* host_buf, int64_t host_bytes,
                                const int64_t* slice_bytes, int32_t n_slices, int32_t scrub) {
  if (!c || n_slices < 0 || (n_slices > 0 && (!slice_bytes || !host_buf || sync_ns < 0)))
    return pf::fail(PF_ERR_ARG, "pf_ctx_set_main_offload: bad argument");
  if (!c->tr || c->md.vocab != 0)
    return pf::fail(PF_ERR_STATE, "pf_ctx_set_main_offload: needs a training context without vocabulary");
  int64_t total = 0;
  for (int32_t j = 0; j < n_slices; ++j) {
    if (slice_bytes[j] < 0 || slice_bytes[j] % 4 != 0)
      return pf::fail(PF_ERR_ARG, "pf_ctx_set_main_offload: slice %d has %lld bytes (must be >= 0 and a multiple of 4)", j,
                      (long long)slice_bytes[j]);
    total += slice_bytes[j];
    if (total > pf::train_opt_state_bytes(c))
      return pf::fail(PF_ERR_ARG, "pf_ctx_set_main_offload: the slices exceed the optimizer state of %lld bytes",
                      (long long)pf::train_opt_state_bytes(c));
  }
  if (total > host_bytes)
    return pf::fail(PF_ERR_CAPACITY, "pf_ctx_set_main_offload: %lld host bytes needed", (long long)total);
  PF_HIP(hipDeviceSynchronize());
  if (n_slices > 0 && !c->off.stream) PF_HIP(hipStreamCreateWithFlags(&c->off.stream, hipStreamNonBlocking));
  c->off.opt_phase = sync_ns >= 0;
  c->off.sync_ns = sync_ns >= 0 ? sync_ns : 0;
  c->off.host = (char*)host_buf;
  c->off.slices.assign(slice_bytes, slice_bytes + n_slices);
  c->off.scrub = scrub != 0;
  return PF_OK;
}

int32_t pf_timeline_run(pf_ctx* fc, pf_ctx* mc, const void* main_io, int32_t p, int32_t m, int32_t stage,
                        int64_t tf_ns, int64_t tb_ns, const pf_bubble* W, int32_t nW, const pf_chunk* plan,
                        int32_t n_plan, const pf_node* F, int32_t nF, int32_t* cursor, void* fill_stream,
                        void* main_stream, pf_timeline_stats* stats) {
  const bool explicit_cycle = (p == 0);   // windows given with their own start times, main stage is a placeholder
  if (explicit_cycle) {
    if (mc || nW <= 0 || !W || !stats) return pf::fail(PF_ERR_ARG, "pf_timeline_run: bad explicit cycle");
    int64_t t = 0;
    for (int32_t k = 0; k < nW; ++k) {
      if (W[k].start_ns < t || W[k].dur_ns <= 0) return pf::fail(PF_ERR_ARG, "pf_timeline_run: windows overlap or are empty");
      t = W[k].start_ns + W[k].dur_ns;
    }
  } else if (p < 1 || m < 1 || stage < 0 || stage >= p || tf_ns <= 0 || tb_ns <= 0 || nW < 0 || (nW > 0 && !W) || !stats)
    return pf::fail(PF_ERR_ARG, "pf_timeline_run: bad schedule argument");
  if (fc && fc->replan && !fc->active_plan.empty()) {   // the plan of the fill job now running
    plan = fc->active_plan.data();
    n_plan = (int32_t)fc->active_plan.size();
  }
  if (fc && (!plan || n_plan <= 0 || !F || nF <= 0 || !cursor || *cursor < 0 || *cursor >= n_plan))
    return pf::fail(PF_ERR_ARG, "pf_timeline_run: bad plan argument");
  hipStream_t fs = (hipStream_t)fill_stream, mstr = (hipStream_t)main_stream;
  if (fc && fs == mstr) return pf::fail(PF_ERR_ARG, "pf_timeline_run: fill and main streams must differ");
  // instruction list of the stage in 1F1B order, bubbles where the schedule has idle windows
  struct Instr { int32_t kind, index; };
  constexpr int32_t INSTR_WAIT = 100;   // explicit cycle: the closed interval before window `index`
  constexpr int32_t INSTR_SYNC = 101;   // main stage: gradient synchronisation, the optimizer state comes back meanwhile
  std::vector<Instr> prog;
  if (explicit_cycle) {
    for (int32_t k = 0; k < nW; ++k) {
      prog.push_back({INSTR_WAIT, k});
      prog.push_back({PF_INSTR_BUBBLE, k});
    }
  }
  const int32_t nf0 = explicit_cycle ? 0 : std::min(p - stage, m);
  const bool has_fb = (int64_t)p * tf_ns + (int64_t)(p - 1 - stage) * tb_ns > (int64_t)(stage + nf0) * tf_ns;
  int32_t nb = 0;
  for (int32_t j = 0; j < nf0; ++j) prog.push_back({PF_INSTR_FWD, j});
  if (has_fb && !explicit_cycle) prog.push_back({PF_INSTR_BUBBLE, nb++});
  int32_t fnext = nf0;
  bool fwd_before = true;
  for (int32_t j = 0; j < m && !explicit_cycle; ++j) {
    if (!fwd_before) prog.push_back({PF_INSTR_BUBBLE, nb++});
    prog.push_back({PF_INSTR_BWD, j});
    fwd_before = false;
    if (fnext < m) {
      prog.push_back({PF_INSTR_FWD, fnext++});
      fwd_before = true;
    }
  }
  if (mc && mc->cfg.g < std::min(p - stage, m))
    return pf::fail(PF_ERR_ARG, "pf_timeline_run: stage %d of %d keeps %d microbatches in flight, the main context has "
                    "checkpoint slots for %d", stage, p, std::min(p - stage, m), mc->cfg.g);
  const bool opt_phase = mc && mc->off.opt_phase;
  const bool offload = opt_phase && !mc->off.slices.empty();
  if (offload && (int32_t)mc->off.slices.size() != m)
    return pf::fail(PF_ERR_ARG, "pf_timeline_run: the main stage has %d offload slices for %d forwards",
                    (int32_t)mc->off.slices.size(), m);
  if (opt_phase) {   // after the last backward: gradient synchronisation, then the optimizer update
    prog.push_back({INSTR_SYNC, 0});
    prog.push_back({PF_INSTR_OPT, m});
  }
  if (stage > 0 && !explicit_cycle) prog.push_back({PF_INSTR_BUBBLE, nb++});
  if (!explicit_cycle && nb != nW)
    return pf::fail(PF_ERR_ARG, "pf_timeline_run: the schedule has %d idle windows, %d were passed", nb, nW);

  std::memset(stats, 0, sizeof *stats);
  struct Rec { hipEvent_t fs0, fs1, dead; bool used; };
  std::vector<Rec> recs(nW, Rec{nullptr, nullptr, nullptr, false});
  hipStream_t tstream = nullptr;   // idle stream: an event recorded on it is stamped "now"
  int32_t rc = PF_OK;
  auto hipck = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && rc == PF_OK) rc = pf::fail(PF_ERR_HIP, "pf_timeline_run: %s: %s", what, hipGetErrorString(e));
    return e == hipSuccess;
  };
  hipck(hipStreamCreateWithFlags(&tstream, hipStreamNonBlocking), "stream");
  for (auto& r : recs) {
    hipck(hipEventCreate(&r.fs0), "event");
    hipck(hipEventCreate(&r.fs1), "event");
    hipck(hipEventCreate(&r.dead), "event");
  }
  double main_ms = 0.0;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> main_ev;
  const int64_t t_start = now_ns();
  int64_t t_sched = t_start;          // scheduled time of the next instruction (placeholder main stage)
  int64_t gone = 0, scrubbed = 0;     // bytes of the main job's optimizer state off the device / overwritten there
  for (size_t pc = 0; pc < prog.size() && rc == PF_OK; ++pc) {
    const Instr in = prog[pc];
    if (in.kind == INSTR_WAIT) {
      const int64_t prev_end = in.index ? W[in.index - 1].start_ns + W[in.index - 1].dur_ns : 0;
      t_sched += W[in.index].start_ns - prev_end;
      wait_until(t_sched);
      continue;
    }
    if (in.kind == INSTR_SYNC) {
      hipck(hipStreamSynchronize(mstr), "main sync");
      const int64_t t0 = now_ns();
      if (offload && gone > 0 && rc == PF_OK) rc = pf::train_opt_state_copy(mc, 0, gone, mc->off.host, false, mc->off.stream);
      wait_until(t0 + mc->off.sync_ns);
      if (offload) {   // the optimizer update needs the state: whatever is still on its way holds the main job up
        const int64_t t1 = now_ns();
        hipck(hipStreamSynchronize(mc->off.stream), "offload sync");
        stats->offload_wait_ns += now_ns() - t1;
        stats->offloaded_bytes = gone;
        gone = scrubbed = 0;
      }
      continue;
    }
    if (in.kind != PF_INSTR_BUBBLE) {
      if (mc && offload && in.kind == PF_INSTR_FWD && mc->off.slices[in.index] > 0 && rc == PF_OK) {
        // this forward's slice of the optimizer state leaves on the copies' stream while the forward runs
        rc = pf::train_opt_state_copy(mc, gone, mc->off.slices[in.index], mc->off.host, true, mc->off.stream);
        gone += mc->off.slices[in.index];
      }
      if (mc) {
        hipEvent_t a = nullptr, b = nullptr;
        hipck(hipEventCreate(&a), "event");
        hipck(hipEventCreate(&b), "event");
        main_ev.push_back({a, b});
        if (rc == PF_OK) hipck(hipEventRecord(a, mstr), "record");
        if (rc == PF_OK) rc = pf_main_stage_step(mc, in.kind, in.index, main_io, main_stream);
        if (rc == PF_OK) hipck(hipEventRecord(b, mstr), "record");
      } else {
        t_sched += (in.kind == PF_INSTR_FWD) ? tf_ns : tb_ns;
        wait_until(t_sched);
      }
      continue;
    }
    const pf_bubble& w = W[in.index];
    // the bubble opens when the stage has nothing left to run
    if (mc) {
      hipck(hipStreamSynchronize(mstr), "main sync");
      if (offload) {   // copies still under way are waited for before the Executor is signalled
        const int64_t t0 = now_ns();
        hipck(hipStreamSynchronize(mc->off.stream), "offload sync");
        stats->offload_wait_ns += now_ns() - t0;
        if (mc->off.scrub && gone > scrubbed && rc == PF_OK) {
          rc = pf::train_opt_state_fill(mc, scrubbed, gone - scrubbed, 0xff, mc->off.stream);
          scrubbed = gone;
        }
      }
      t_sched = now_ns();
    }
    const int64_t deadline = t_sched + w.dur_ns;
    stats->idle_ns += w.dur_ns;
    if (w.fillable) stats->offered_ns += w.dur_ns;
    if (rc == PF_OK && fc && w.fillable && plan[*cursor].bubble == in.index) {
      int64_t planned_ns = 0;   // planned duration of the chunks already launched in this window
      for (bool again = true; again && rc == PF_OK;) {
        again = false;
        const pf_chunk ch = plan[*cursor];
        if (ch.node_end > ch.node_begin) {
          Rec& r = recs[in.index];
          if (!r.used) hipck(hipEventRecord(r.fs0, fs), "record");
          if (rc == PF_OK) rc = pf_fill_chunk(fc, &ch, F, nF, w.free_bytes, fill_stream);
          if (rc == PF_OK) hipck(hipEventRecord(r.fs1, fs), "record");
          r.used = r.used || (rc == PF_OK);
          stats->chunks_run += 1;
          for (int32_t j = ch.node_begin; j < ch.node_end; ++j)
            if (j % nF == nF - 1) stats->replicas_done += 1;
        }
        planned_ns += ch.dur_ns;
        if (++*cursor < n_plan) break;
        *cursor = 0;
        fc->replica_base += plan[n_plan - 1].node_end / nF;
        if (!fc->replan || rc != PF_OK) break;
        // The job is complete.  The next one starts in what is left of this window: its duration less the
        // share already planned (which charges the new job its own switch time).
        int32_t ord = 0;
        for (int32_t k = 0; k <= in.index; ++k) ord += W[k].fillable ? 1 : 0;
        int64_t left = 0;
        if (fc->replan_ppm > 0) {
          const __int128 spent = ((__int128)planned_ns * 1000000 + fc->replan_ppm - 1) / fc->replan_ppm;
          left = spent < w.dur_ns ? w.dur_ns - (int64_t)spent : 0;
        }
        std::vector<pf_chunk> next;
        int32_t n_new = 0;
        int32_t prc = pf_plan_bubbles_from(W, nW, F, nF, fc->replan_ppm, fc->replan_switch_ns, ord - 1, left, nullptr, 0,
                                           &n_new, nullptr);
        if (prc == PF_ERR_CAPACITY || prc == PF_OK) {
          next.resize((size_t)n_new);
          prc = pf_plan_bubbles_from(W, nW, F, nF, fc->replan_ppm, fc->replan_switch_ns, ord - 1, left, next.data(),
                                     n_new, &n_new, nullptr);
        }
        if (prc == PF_OK && n_new <= 0) prc = pf::fail(PF_ERR_STATE, "pf_timeline_run: empty plan");
        if (prc != PF_OK) {
          rc = prc;
        } else {
          fc->active_plan.swap(next);
          plan = fc->active_plan.data();
          n_plan = n_new;
          again = true;   // its first chunk belongs to this window
        }
      }
    }
    wait_until(deadline);
    if (rc == PF_OK && recs[in.index].used) hipck(hipEventRecord(recs[in.index].dead, tstream), "record");
    t_sched = deadline;
  }
  hipck(hipDeviceSynchronize(), "final sync");
  stats->iter_ns = (mc ? now_ns() : t_sched) - t_start;
  if (rc == PF_OK) {
    for (auto& r : recs) {
      if (!r.used) continue;
      float busy = 0.f, over = 0.f;
      hipck(hipEventElapsedTime(&busy, r.fs0, r.fs1), "elapsed");
      hipck(hipEventElapsedTime(&over, r.dead, r.fs1), "elapsed");
      stats->fill_busy_ns += (int64_t)(busy * 1e6);
      if (over > 0.f) stats->overrun_ns += (int64_t)(over * 1e6);
    }
    for (auto& pr : main_ev) {
      float t = 0.f;
      hipck(hipEventElapsedTime(&t, pr.first, pr.second), "elapsed");
      main_ms += t;
    }
    stats->main_busy_ns = (int64_t)(main_ms * 1e6);
  }
  for (auto& r : recs) {
    if (r.fs0) (void)hipEventDestroy(r.fs0);
    if (r.fs1) (void)hipEventDestroy(r.fs1);
    if (r.dead) (void)hipEventDestroy(r.dead);
  }
  for (auto& pr : main_ev) {
    if (pr.first) (void)hipEventDestroy(pr.first);
    if (pr.second) (void)hipEventDestroy(pr.second);
  }
  if (tstream) (void)hipStreamDestroy(tstream);
  return rc;
}

int32_t pf_probe_bubbles_live(pf_ctx* mc, const void* main_io, int32_t p, int32_t m, int32_t stage, int64_t tf_ns,
                              int64_t tb_ns, int64_t first_wait_ns, int64_t tol_ppm, int64_t* est_ns, int32_t cap,
                              int32_t* n_out, int64_t* base_period_ns, void* main_stream) {
  if (!mc || !main_io || p < 1 || m < 1 || stage < 0 || stage >= p || tf_ns <= 0 || tb_ns <= 0 || first_wait_ns < 1 ||
      tol_ppm < 0 || cap < 0 || !n_out || (cap > 0 && !est_ns) || (int64_t)p * m > (int64_t)1 << 16)
    return pf::fail(PF_ERR_ARG, "pf_probe_bubbles_live: bad argument");
  if (!mc->tr || mc->md.vocab != 0)
    return pf::fail(PF_ERR_STATE, "pf_probe_bubbles_live: needs a training context without vocabulary");
  if (mc->cfg.g < std::min(p - stage, m))
    return pf::fail(PF_ERR_ARG, "pf_probe_bubbles_live: stage %d of %d keeps %d microbatches in flight, the main context has "
                    "checkpoint slots for %d", stage, p, std::min(p - stage, m), mc->cfg.g);
  std::vector<std::vector<pf::StageOp>> ops;
  for (int32_t q = 0; q < p; ++q) ops.push_back(pf::stage_ops(p, m, q));
  int32_t n = 0;
  for (const pf::StageOp& o : ops[stage]) n += (o.op == 2);
  *n_out = n;
  if (n > cap) return pf::fail(PF_ERR_CAPACITY, "pf_probe_bubbles_live: %d windows, capacity %d", n, cap);
  hipStream_t st = (hipStream_t)main_stream;
  int32_t rc = PF_OK;
  // One trial = four iterations of the pipeline: the other stages are simulated from tf_ns / tb_ns, this stage's
  // instructions run on the device when the simulation says their inputs have arrived (never earlier than the
  // wall clock allows), and their measured finish times go back into the simulation.
  auto trial = [&](const std::vector<int64_t>& waits) -> int64_t {
    (void)hipStreamSynchronize(st);
    const int64_t origin = now_ns();
    return pf::period_with_waits(p, m, tf_ns, tb_ns, stage, waits, ops, [&](int32_t op, int32_t idx, int64_t start) -> int64_t {
      wait_until(origin + start);
      rc = pf_main_stage_step(mc, op == 0 ? PF_INSTR_FWD : PF_INSTR_BWD, idx, main_io, main_stream);
      if (rc != PF_OK) return -1;
      if (hipStreamSynchronize(st) != hipSuccess) {
        rc = pf::fail(PF_ERR_HIP, "pf_probe_bubbles_live: stream synchronisation failed");
        return -1;
      }
      return now_ns() - origin;
    });
  };
  std::vector<int64_t> waits(n, 0);
  (void)trial(waits);   // warm-up
  int64_t base = trial(waits);
  if (base >= 0) base = std::min(base, trial(waits));
  if (base < 0) return rc;
  if (base_period_ns) *base_period_ns = base;
  const int64_t limit = base + (int64_t)((__int128)base * tol_ppm / 1000000);
  for (int32_t k = 0; k < n; ++k) {
    int64_t w = first_wait_ns;
    for (;;) {
      const int64_t keep = waits[k];
      waits[k] = w;
      const int64_t per = trial(waits);
      if (per < 0) return rc;
      if (per > limit || w > base) {   // a wait longer than a whole iteration cannot be harmless
        waits[k] = keep;
        break;
      }
      w *= 2;
    }
  }
  for (int32_t k = 0; k < n; ++k) est_ns[k] = waits[k];
  return PF_OK;
}

int32_t pf_ctx_set_replan(pf_ctx* c, int32_t enable, int64_t fill_ppm, int64_t switch_ns) {
  if (!c || fill_ppm < 0 || fill_ppm > 1000000 || switch_ns < 0)
    return pf::fail(PF_ERR_ARG, "pf_ctx_set_replan: bad argument");
  c->replan = enable != 0;
  c->replan_ppm = fill_ppm;
  c->replan_switch_ns = switch_ns;
  c->active_plan.clear();
  return PF_OK;
}

int32_t pf_ctx_train_state(pf_ctx* c, double* loss, int64_t* steps) {
  if (!c) return pf::fail(PF_ERR_ARG, "pf_ctx_train_state: null context");
  if (!c->tr) return pf::fail(PF_ERR_STATE, "pf_ctx_train_state: not a training context");
  PF_HIP(hipDeviceSynchronize());
  if (steps) *steps = c->tr->steps;
  if (loss) {
    float sum = 0.f;
    PF_HIP(hipMemcpy(&sum, c->tr->loss, sizeof sum, hipMemcpyDeviceToHost));
    PF_HIP(hipMemset(c->tr->loss, 0, sizeof sum));
    const double n = (double)c->tr->loss_count * c->md.batch * (c->md.seq_len - 1);
    *loss = n > 0 ? sum / n : 0.0;
    c->tr->loss_count = 0;
  }
  return PF_OK;
}

int32_t pf_ctx_read_params(pf_ctx* c, int32_t what, int32_t layer, void* dst, int64_t dst_bytes, void* stream) {
  if (!c || !dst || what < 0 || what > 3 || layer < -1)
    return pf::fail(PF_ERR_ARG, "pf_ctx_read_params: bad argument");
  if (!c->tr) return pf::fail(PF_ERR_STATE, "pf_ctx_read_params: not a training context");
  return pf::train_read_params(c, what, layer, dst, dst_bytes, (hipStream_t)stream);
}

int32_t pf_ctx_kernel_timing(pf_ctx* c, uint32_t mask) {
  if (!c) return pf::fail(PF_ERR_ARG, "pf_ctx_kernel_timing: null context");
  if (mask && c->timing_pool.empty()) {
    c->timing_pool.resize(16384);
    for (auto& p : c->timing_pool) {
      p.a = p.b = nullptr;
      PF_HIP(hipEventCreate(&p.a));
      PF_HIP(hipEventCreate(&p.b));
    }
  }
  int32_t rc = drain_timing(c);
  if (rc != PF_OK) return rc;
  for (int i = 0; i < PF_KERNEL_CLASSES; ++i) {
    c->cls_count[i] = 0;
    c->cls_ms[i] = 0.0;
  }
  c->timing_mask = mask;
  return PF_OK;
}

int32_t pf_ctx_kernel_timing_every(pf_ctx* c, int32_t n) {
  if (!c || n < 1) return pf::fail(PF_ERR_ARG, "pf_ctx_kernel_timing_every: bad argument");
  c->timing_every = n;
  for (int i = 0; i < PF_KERNEL_CLASSES; ++i) c->cls_seen[i] = 0;
  return PF_OK;
}

int32_t pf_ctx_kernel_stats(pf_ctx* c, int32_t cls, int64_t* count, int64_t* total_ns) {
  if (!c || cls < 0 || cls >= PF_KERNEL_CLASSES || !count || !total_ns)
    return pf::fail(PF_ERR_ARG, "pf_ctx_kernel_stats: bad argument");
  int32_t rc = drain_timing(c);
  if (rc != PF_OK) return rc;
  *count = c->cls_count[cls];
  *total_ns = (int64_t)(c->cls_ms[cls] * 1e6);
  return PF_OK;
}

// ---- single kernels --------------------------------------------------------------------------------
static bool bad_dtype(int32_t dt) { return dt != PF_DTYPE_F32 && dt != PF_DTYPE_BF16; }

int32_t pf_op_gemm(int32_t dtype, const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K,
                   const void* bias, const void* resid, int32_t gelu, int32_t out_f32, int32_t accumulate,
                   const void* dact_in, void* preact_out, void* stream) {
  if (bad_dtype(dtype) || !X || !W || !C || M <= 0 || N <= 0 || K <= 0 || (dtype == PF_DTYPE_BF16 && K % 8 != 0) ||
      (accumulate && !out_f32 && dtype != PF_DTYPE_F32) ||
      (dact_in && (bias || resid || gelu || preact_out || out_f32)) || (preact_out && out_f32))
    return pf::fail(PF_ERR_ARG, "pf_op_gemm: bad argument");
  pf::GemmEpilogue e;
  e.bias = bias;
  e.resid = resid;
  e.gelu = gelu;
  e.out_f32 = out_f32;
  e.accumulate = accumulate;
  e.dact_in = dact_in;
  e.preact_out = preact_out;
  PF_HIP(pf::gemm_nt(dtype, X, W, C, M, N, K, e, (hipStream_t)stream));
  return PF_OK;
}

int32_t pf_op_layernorm(int32_t dtype, const void* x, const void* g, const void* b, void* y, float* mean_out,
                        float* rstd_out, int64_t rows, int32_t d, float eps, const void* warm, int64_t warm_bytes,
                        void* stream) {
  if (bad_dtype(dtype) || !x || !g || !b || !y || rows <= 0 || d <= 0 || d % 8 != 0 || d > 8192 || warm_bytes < 0)
    return pf::fail(PF_ERR_ARG, "pf_op_layernorm: bad argument (d must be a multiple of 8, at most 8192)");
  PF_HIP(pf::layernorm_fwd(dtype, x, g, b, y, mean_out, rstd_out, rows, d, eps, (hipStream_t)stream, warm, warm_bytes));
  return PF_OK;
}

int32_t pf_op_attention(int32_t dtype, const void* qkv, void* out, float* lse, int32_t B, int32_t S, int32_t h,
                        int32_t dh, int32_t causal, void* stream) {
  if (bad_dtype(dtype) || !qkv || !out || B <= 0 || S <= 0 || h <= 0 || B > 65535 || h > 65535 ||
      !(dh == 8 || dh == 16 || dh == 32 || dh == 64 || dh == 128))
    return pf::fail(PF_ERR_ARG, "pf_op_attention: bad argument (d_head must be 8, 16, 32, 64 or 128)");
  PF_HIP(pf::attention_fwd(dtype, qkv, out, lse, B, S, h, dh, causal, (hipStream_t)stream));
  return PF_OK;
}

int32_t pf_op_attention_bwd(int32_t dtype, const void* qkv, const void* out, const void* dout, const float* lse,
                            float* dsum, void* dqkv, int32_t B, int32_t S, int32_t h, int32_t dh, int32_t causal,
                            void* stream) {
  if (bad_dtype(dtype) || !qkv || !out || !dout || !lse || !dsum || !dqkv || B <= 0 || S <= 0 || h <= 0 || B > 65535 ||
      h > 65535 || !(dh == 8 || dh == 16 || dh == 32 || dh == 64 || dh == 128))
    return pf::fail(PF_ERR_ARG, "pf_op_attention_bwd: bad argument");
  PF_HIP(pf::attention_bwd(dtype, qkv, out, dout, lse, dsum, dqkv, B, S, h, dh, causal, (hipStream_t)stream));
  return PF_OK;
}

int32_t pf_op_layernorm_bwd(int32_t dtype, const void* dy, const void* x, const void* g, const float* mean,
                            const float* rstd, const void* resid, void* dx, float* dg, float* db, float* partial,
                            int64_t rows, int32_t d, void* stream) {
  if (bad_dtype(dtype) || !dy || !x || !g || !mean || !rstd || !dx || !dg || !db || !partial || rows <= 0 || d <= 0 ||
      d % 8 != 0 || d > 8192)
    return pf::fail(PF_ERR_ARG, "pf_op_layernorm_bwd: bad argument");
  PF_HIP(pf::layernorm_bwd(dtype, dy, x, g, mean, rstd, resid, dx, dg, db, partial, rows, d, (hipStream_t)stream));
  return PF_OK;
}

int32_t pf_op_transpose(int32_t dtype, const void* in, void* out, int64_t rows, int64_t cols, float* colsum_acc,
                        void* stream) {
  if (bad_dtype(dtype) || !in || !out || in == out || rows <= 0 || cols <= 0 || (rows + 63) / 64 > 65535)
    return pf::fail(PF_ERR_ARG, "pf_op_transpose: bad argument");
  if (colsum_acc) PF_HIP(pf::transpose2d_colsum(dtype, in, out, colsum_acc, rows, cols, (hipStream_t)stream));
  else PF_HIP(pf::transpose2d(dtype, in, out, rows, cols, (hipStream_t)stream));
  return PF_OK;
}

int32_t pf_op_gemm_tn(int32_t dtype, const void* A, const void* B, float* C, float* colsum_acc, int64_t M, int64_t N,
                      int64_t K, void* stream) {
  if (bad_dtype(dtype) || !A || !B || !C || M <= 0 || N <= 0 || K <= 0)
    return pf::fail(PF_ERR_ARG, "pf_op_gemm_tn: bad argument");
  if (!pf::gemm_tn_acc_supported(dtype, A, B, M, N, K))
    return pf::fail(PF_ERR_ARG, "pf_op_gemm_tn: needs bf16, M and N multiples of 8, K a multiple of 64, 16-byte aligned operands");
  PF_HIP(pf::gemm_tn_acc(dtype, A, B, C, colsum_acc, M, N, K, (hipStream_t)stream));
  return PF_OK;
}

int32_t pf_op_embed(int32_t dtype, const int32_t* ids, const void* tok, const void* pos, void* x, int64_t tokens,
                    int32_t S, int32_t d, int32_t V, void* stream) {
  if (bad_dtype(dtype) || !ids || !tok || !pos || !x || tokens <= 0 || S <= 0 || d <= 0 || d % 8 != 0 || V <= 0)
    return pf::fail(PF_ERR_ARG, "pf_op_embed: bad argument");
  PF_HIP(pf::embed_fwd(dtype, ids, tok, pos, x, tokens, S, d, V, (hipStream_t)stream));
  return PF_OK;
}

}  // extern "C"
