// Training fill jobs and the emulated main-job stage: parameter state (fp32 master weights, Adam
// moments, gradient accumulators, working and transposed copies in the model dtype), layer backward
// with recompute from the layer's checkpoint, tied-head loss, embedding backward and Adam.
//
// Forward and dX GEMMs run on the "NT" kernel (both operands contiguous along the contraction):
//   dX = dY * W      uses the transposed weight copy kept next to the working weights.
// Weight gradients dW += dY^T * X contract over tokens, the slow index of both tensors: in bf16 the "TN"
// kernel reads them as they are (and sums dY's columns for the bias gradient on the way); in fp32 transposes
// of the two tensors, made just before, feed the NT kernel.  Either way fp32 accumulation goes straight into
// the gradient accumulators.
#include <cstring>
#include <new>

#include "pf_kernels.h"
#include "pf_runtime.h"

#define PF_HIP(expr)                                                                              \
  do {                                                                                            \
    hipError_t e__ = (expr);                                                                      \
    if (e__ != hipSuccess)                                                                        \
      return pf::fail(PF_ERR_HIP, "%s: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
  } while (0)

namespace pf {

namespace {

// rows / columns of the 12 parameter arrays of a layer (vectors are 1 x n)
void param_shape(const pf_model_desc& m, int i, int64_t* R, int64_t* C) {
  const int64_t d = m.d_model, f = m.d_ff;
  switch (i) {
    case 2: *R = 3 * d; *C = d; break;
    case 3: *R = 1; *C = 3 * d; break;
    case 4: *R = d; *C = d; break;
    case 8: *R = f; *C = d; break;
    case 9: *R = 1; *C = f; break;
    case 10: *R = d; *C = f; break;
    default: *R = 1; *C = d; break;
  }
}
const int kMat[4] = {2, 4, 8, 10};   // w_qkv, w_o, w_1, w_2

struct Sizes {
  int64_t e, T, d, f, act, mid, blob32, off32[12], wt_off[4], wt, Vp, embw_tok, embw_pos, embw_vec, emb32_off[4],
      emb32, lse, stat, tA, lnp, logits;
};

Sizes sizes_of(const pf_model_desc& m, const Layout& lay) {
  Sizes z{};
  z.e = lay.esz;
  z.T = lay.tokens;
  z.d = m.d_model;
  z.f = m.d_ff;
  z.act = lay.act;
  z.mid = align_up(z.T * z.f * z.e, 256);
  int64_t o = 0;
  for (int i = 0; i < 12; ++i) {
    int64_t R, C;
    param_shape(m, i, &R, &C);
    z.off32[i] = o;
    o += align_up(R * C * 4, 256);
  }
  z.blob32 = o;
  o = 0;
  for (int k = 0; k < 4; ++k) {
    int64_t R, C;
    param_shape(m, kMat[k], &R, &C);
    z.wt_off[k] = o;
    o += align_up(R * C * z.e, 256);
  }
  z.wt = o;
  z.Vp = m.vocab > 0 ? align_up(m.vocab, 64) : 0;
  if (z.Vp) {
    z.embw_tok = align_up(z.Vp * z.d * z.e, 256);
    z.embw_pos = align_up((int64_t)m.seq_len * z.d * z.e, 256);
    z.embw_vec = align_up(z.d * z.e, 256);
    z.emb32_off[0] = 0;
    z.emb32_off[1] = align_up(z.Vp * z.d * 4, 256);
    z.emb32_off[2] = z.emb32_off[1] + align_up((int64_t)m.seq_len * z.d * 4, 256);
    z.emb32_off[3] = z.emb32_off[2] + align_up(z.d * 4, 256);
    z.emb32 = z.emb32_off[3] + align_up(z.d * 4, 256);
    z.logits = align_up(z.T * z.Vp * z.e, 256);
  }
  z.lse = align_up((int64_t)m.batch * m.n_heads * m.seq_len * 4, 256);
  z.stat = align_up(z.T * 4, 256);
  const int64_t ta_elems = (z.T * z.f > 3 * z.T * z.d) ? z.T * z.f : 3 * z.T * z.d;
  z.tA = align_up(ta_elems * z.e, 256);
  z.lnp = align_up(LN_BWD_MAX_BLOCKS * 4 * 2 * z.d * 4, 256);
  return z;
}

}  // namespace

int64_t train_arena_bytes(const pf_model_desc& m, const pf_exec_config& cfg, const Layout& lay) {
  const Sizes z = sizes_of(m, lay);
  const int64_t L = m.n_layers, g = cfg.g;
  int64_t t = 0;
  t += L * (lay.blob + z.wt + 4 * z.blob32);                                  // per-layer parameter state
  if (z.Vp) t += 2 * z.embw_tok + z.embw_pos + 2 * z.embw_vec + 4 * z.emb32;  // embeddings, final LayerNorm
  t += g * (L + 1) * z.act + g * z.act + (z.Vp ? g * z.act : 0);              // checkpoints, gradients, head input
  t += 2 * z.act + z.mid + 2 * z.lse + 6 * z.stat;                            // ln2, x1, u, lse, Dsum, statistics
  t += z.mid + 3 * z.act + 2 * z.act + z.tA + z.mid + z.lnp;                  // d_mid, d_qkv, d_attn, d_ln, tA, tB
  if (z.Vp) t += 2 * z.logits;
  t += 256;
  return t;
}

static int32_t recast_layer(pf_ctx* c, int32_t l, hipStream_t st) {
  TrainState& t = *c->tr;
  for (int i = 0; i < 12; ++i) {
    int64_t R, C;
    param_shape(c->md, i, &R, &C);
    void* dst_t = nullptr;
    for (int k = 0; k < 4; ++k)
      if (kMat[k] == i) dst_t = t.Wt[l] + t.wt_off[k];
    PF_HIP(cast_from_f32(c->md.dtype, (const float*)((char*)t.master[l] + t.off32[i]), t.Wk[l] + c->lay.off[i], dst_t,
                         R, C, st));
  }
  return PF_OK;
}

static int32_t recast_emb(pf_ctx* c, hipStream_t st) {
  TrainState& t = *c->tr;
  const pf_model_desc& m = c->md;
  PF_HIP(cast_from_f32(m.dtype, (const float*)((char*)t.embM + t.emb32_off[0]), t.E_w, t.Et, t.Vp, m.d_model, st));
  PF_HIP(cast_from_f32(m.dtype, (const float*)((char*)t.embM + t.emb32_off[1]), t.pos_w, nullptr, m.seq_len, m.d_model, st));
  PF_HIP(cast_from_f32(m.dtype, (const float*)((char*)t.embM + t.emb32_off[2]), t.lnf_g_w, nullptr, 1, m.d_model, st));
  PF_HIP(cast_from_f32(m.dtype, (const float*)((char*)t.embM + t.emb32_off[3]), t.lnf_b_w, nullptr, 1, m.d_model, st));
  return PF_OK;
}

int32_t train_create(pf_ctx* c, const pf_weights* w, char* base, hipStream_t st) {
  TrainState* tp = new (std::nothrow) TrainState();
  if (!tp) return fail(PF_ERR_NOMEM, "pf_ctx_create: host allocation failed");
  c->tr = tp;
  TrainState& t = *tp;
  const pf_model_desc& m = c->md;
  const Sizes z = sizes_of(m, c->lay);
  const int64_t L = m.n_layers, g = c->cfg.g;
  t.Vp = z.Vp;
  t.blob32 = z.blob32;
  std::memcpy(t.off32, z.off32, sizeof z.off32);
  std::memcpy(t.wt_off, z.wt_off, sizeof z.wt_off);
  std::memcpy(t.emb32_off, z.emb32_off, sizeof z.emb32_off);
  t.wt_bytes = z.wt;
  t.emb32 = z.emb32;
  t.slot_live.assign((size_t)g, 0);
  char* p = base;
  auto take = [&](int64_t n) { char* r = p; p += n; return r; };
  for (int64_t l = 0; l < L; ++l) {
    t.Wk.push_back(take(c->lay.blob));
    t.Wt.push_back(take(z.wt));
    t.master.push_back((float*)take(z.blob32));
    t.m.push_back((float*)take(z.blob32));
    t.v.push_back((float*)take(z.blob32));
    t.grad.push_back((float*)take(z.blob32));
  }
  if (z.Vp) {
    t.E_w = take(z.embw_tok);
    t.Et = take(z.embw_tok);
    t.pos_w = take(z.embw_pos);
    t.lnf_g_w = take(z.embw_vec);
    t.lnf_b_w = take(z.embw_vec);
    t.embM = (float*)take(z.emb32);
    t.embm = (float*)take(z.emb32);
    t.embv = (float*)take(z.emb32);
    t.embg = (float*)take(z.emb32);
  }
  t.ckpt = take(g * (L + 1) * z.act);
  t.G = take(g * z.act);
  if (z.Vp) t.Hf = take(g * z.act);
  t.ln2 = take(z.act);
  t.x1 = take(z.act);
  t.u = take(z.mid);
  t.lse = (float*)take(z.lse);
  t.Dsum = (float*)take(z.lse);
  t.stats = (float*)take(6 * z.stat);
  t.stat_stride = z.stat / 4;
  t.d_mid = take(z.mid);
  t.d_qkv = take(3 * z.act);
  t.d_attn = take(z.act);
  t.d_ln = take(z.act);
  t.tA = take(z.tA);
  t.tB = take(z.mid);
  t.ln_partial = (float*)take(z.lnp);
  if (z.Vp) {
    t.logits = take(z.logits);
    t.logitsT = take(z.logits);
  }
  t.loss = (float*)take(256);

  // parameters: widen the caller's arrays into the master copy, derive the working copies from it
  for (int64_t l = 0; l < L; ++l) {
    PF_HIP(hipMemsetAsync(t.master[l], 0, (size_t)(4 * z.blob32), st));   // master, m, v, grad are adjacent
    for (int i = 0; i < 12; ++i) {
      int64_t R, C;
      param_shape(m, i, &R, &C);
      PF_HIP(widen_to_f32(m.dtype, (const char*)w->layers[l] + c->lay.off[i], (float*)((char*)t.master[l] + z.off32[i]),
                          R * C, st));
    }
    int32_t rc = recast_layer(c, (int32_t)l, st);
    if (rc != PF_OK) return rc;
  }
  if (z.Vp) {
    PF_HIP(hipMemsetAsync(t.embM, 0, (size_t)(4 * z.emb32), st));
    PF_HIP(widen_to_f32(m.dtype, w->tok_emb, (float*)((char*)t.embM + z.emb32_off[0]), (int64_t)m.vocab * m.d_model, st));
    PF_HIP(widen_to_f32(m.dtype, w->pos_emb, (float*)((char*)t.embM + z.emb32_off[1]), (int64_t)m.seq_len * m.d_model, st));
    PF_HIP(widen_to_f32(m.dtype, w->lnf_g, (float*)((char*)t.embM + z.emb32_off[2]), m.d_model, st));
    PF_HIP(widen_to_f32(m.dtype, w->lnf_b, (float*)((char*)t.embM + z.emb32_off[3]), m.d_model, st));
    int32_t rc = recast_emb(c, st);
    if (rc != PF_OK) return rc;
  }
  PF_HIP(hipMemsetAsync(t.loss, 0, 256, st));
  PF_HIP(hipStreamSynchronize(st));
  return PF_OK;
}

void train_destroy(pf_ctx* c) {
  delete c->tr;
  c->tr = nullptr;
}

// ---- layer recompute + backward ---------------------------------------------------------------------
static int32_t layer_backward(pf_ctx* c, int32_t l, const char* x, char* G, hipStream_t st) {
  TrainState& t = *c->tr;
  const pf_model_desc& m = c->md;
  const int64_t* o = c->lay.off;
  const int64_t T = c->lay.tokens;
  const int32_t d = m.d_model, f = m.d_ff, dt = m.dtype, dh = d / m.n_heads;
  const char* wb = t.Wk[l];
  const char* wt = t.Wt[l];
  float* gr = t.grad[l];
  auto G32 = [&](int i) { return (float*)((char*)gr + t.off32[i]); };
  float *mean1 = t.stats, *rstd1 = t.stats + t.stat_stride, *mean2 = t.stats + 2 * t.stat_stride,
        *rstd2 = t.stats + 3 * t.stat_stride;

  // recompute the forward pass, keeping what the backward needs
  PF_HIP(layernorm_fwd(dt, x, wb + o[0], wb + o[1], c->ws_ln, mean1, rstd1, T, d, m.eps, st, wb + o[2],
                       warm_bytes(o[4] - o[2])));                                                                  // a (+ warms W_qkv, b_qkv)
  GemmEpilogue e1;
  e1.bias = wb + o[3];
  PF_HIP(gemm_nt(dt, c->ws_ln, wb + o[2], c->ws_qkv, T, 3 * d, d, e1, st));
  PF_HIP(attention_fwd(dt, c->ws_qkv, c->ws_attn, t.lse, m.batch, m.seq_len, m.n_heads, dh, m.causal, st));  // c
  GemmEpilogue e2;
  e2.bias = wb + o[5];
  e2.resid = x;
  PF_HIP(gemm_nt(dt, c->ws_attn, wb + o[4], t.x1, T, d, d, e2, st));                                      // x1
  PF_HIP(layernorm_fwd(dt, t.x1, wb + o[6], wb + o[7], t.ln2, mean2, rstd2, T, d, m.eps, st, wb + o[8],
                       warm_bytes(o[10] - o[8])));                                                           // bb (+ warms W_1, b_1)
  GemmEpilogue e3;
  e3.bias = wb + o[9];
  e3.gelu = 1;
  e3.preact_out = t.u;
  PF_HIP(gemm_nt(dt, t.ln2, wb + o[8], c->ws_mid, T, f, d, e3, st));                                      // u, gelu(u)

  // y = x1 + gelu(u) W_2 + b_2
  GemmEpilogue b1;
  b1.dact_in = t.u;
  PF_HIP(gemm_nt(dt, G, wt + t.wt_off[3], t.d_mid, T, f, d, b1, st));            // du = (dy W_2) * gelu'(u)
  GemmEpilogue acc;
  acc.out_f32 = 1;
  acc.accumulate = 1;
  // Weight and bias gradient of a linear layer y = x W^T + b from dy [T][n_out] and x [T][n_in]:
  // dW += dy^T x, db += column sums of dy.  bf16: one kernel on the tensors as they are; otherwise transposed
  // copies feed the NT kernel and the column sums come out of the first transpose.
  auto weight_grad = [&](const void* dy, const void* xin, float* dW, float* db, int64_t n_out, int64_t n_in) -> int32_t {
    if (gemm_tn_acc_supported(dt, dy, xin, n_out, n_in, T) && gemm_tn_acc_preferred(n_out, n_in, T)) {
      PF_HIP(gemm_tn_acc(dt, dy, xin, dW, db, n_out, n_in, T, st));
      return PF_OK;
    }
    PF_HIP(transpose2d_colsum(dt, dy, t.tA, db, T, n_out, st));
    PF_HIP(transpose2d(dt, xin, t.tB, T, n_in, st));
    PF_HIP(gemm_nt(dt, t.tA, t.tB, dW, n_out, n_in, T, acc, st));
    return PF_OK;
  };
  int32_t wrc = weight_grad(G, c->ws_mid, G32(10), G32(11), d, f);               // dW_2 [d][f], db_2
  if (wrc != PF_OK) return wrc;
  wrc = weight_grad(t.d_mid, t.ln2, G32(8), G32(9), f, d);                       // dW_1 [f][d], db_1
  if (wrc != PF_OK) return wrc;
  GemmEpilogue none;
  PF_HIP(gemm_nt(dt, t.d_mid, wt + t.wt_off[2], t.d_ln, T, d, f, none, st));     // dbb = du W_1
  PF_HIP(layernorm_bwd(dt, t.d_ln, t.x1, wb + o[6], mean2, rstd2, G, G, G32(6), G32(7), t.ln_partial, T, d, st));
  // G now holds dx1.   x1 = x + c W_o + b_o
  wrc = weight_grad(G, c->ws_attn, G32(4), G32(5), d, d);                        // dW_o [d][d], db_o
  if (wrc != PF_OK) return wrc;
  PF_HIP(gemm_nt(dt, G, wt + t.wt_off[1], t.d_attn, T, d, d, none, st));         // dc = dx1 W_o
  PF_HIP(attention_bwd(dt, c->ws_qkv, c->ws_attn, t.d_attn, t.lse, t.Dsum, t.d_qkv, m.batch, m.seq_len, m.n_heads, dh,
                       m.causal, st));
  wrc = weight_grad(t.d_qkv, c->ws_ln, G32(2), G32(3), 3 * d, d);                // dW_qkv [3d][d], db_qkv
  if (wrc != PF_OK) return wrc;
  PF_HIP(gemm_nt(dt, t.d_qkv, wt + t.wt_off[0], t.d_ln, T, d, 3 * d, none, st)); // da = dqkv W_qkv
  PF_HIP(layernorm_bwd(dt, t.d_ln, x, wb + o[0], mean1, rstd1, G, G, G32(0), G32(1), t.ln_partial, T, d, st));
  return PF_OK;
}

static const int32_t* replica_ids(pf_ctx* c, int64_t replica) {
  if (!c->in || c->n_in <= 0) return nullptr;
  return (const int32_t*)((const char*)c->in + (replica % c->n_in) * ((int64_t)c->cfg.g * c->lay.tokens * 4));
}

int32_t train_fwd_node(pf_ctx* c, const pf_node& n, int64_t replica, hipStream_t st) {
  TrainState& t = *c->tr;
  const pf_model_desc& m = c->md;
  const int64_t act = c->lay.act, T = c->lay.tokens, L = m.n_layers;
  const int32_t g = c->cfg.g, d = m.d_model;
  auto ck = [&](int32_t mb, int64_t l) { return t.ckpt + ((int64_t)mb * (L + 1) + l) * act; };
  switch (n.op) {
    case PF_OP_EMBED: {
      const int32_t* ids = replica_ids(c, replica);
      if (!ids) return fail(PF_ERR_STATE, "training chunk: no input ring set (pf_ctx_set_io)");
      for (int32_t mb = 0; mb < g; ++mb)
        PF_HIP(embed_fwd(m.dtype, ids + mb * T, t.E_w, t.pos_w, ck(mb, 0), T, m.seq_len, d, m.vocab, st));
      return PF_OK;
    }
    case PF_OP_LAYER_FWD:
      for (int32_t mb = 0; mb < g; ++mb) {
        int32_t rc = layer_forward(c, t.Wk[n.layer], ck(mb, n.layer), ck(mb, n.layer + 1), st);
        if (rc != PF_OK) return rc;
      }
      return PF_OK;
    case PF_OP_FINAL_LN:
      if (!t.Vp) return fail(PF_ERR_STATE, "training chunk: FINAL_LN needs a vocabulary");
      for (int32_t mb = 0; mb < g; ++mb)
        PF_HIP(layernorm_fwd(m.dtype, ck(mb, L), t.lnf_g_w, t.lnf_b_w, t.Hf + mb * act, nullptr, nullptr, T, d, m.eps, st));
      return PF_OK;
    case PF_OP_HEAD_LOSS: {
      if (!t.Vp) return fail(PF_ERR_STATE, "training chunk: HEAD_LOSS needs a vocabulary");
      const int32_t* ids = replica_ids(c, replica);
      if (!ids) return fail(PF_ERR_STATE, "training chunk: no input ring set (pf_ctx_set_io)");
      float *meanf = t.stats + 4 * t.stat_stride, *rstdf = t.stats + 5 * t.stat_stride;
      float* ge = t.embg;
      const float inv_n = 1.0f / (float)((int64_t)m.batch * (m.seq_len - 1));
      for (int32_t mb = 0; mb < g; ++mb) {
        char* hf = t.Hf + mb * act;
        GemmEpilogue none;
        PF_HIP(gemm_nt(m.dtype, hf, t.E_w, t.logits, T, t.Vp, d, none, st));                    // logits [T][Vp]
        PF_HIP(ce_loss_inplace(m.dtype, t.logits, ids + mb * T, t.loss, T, t.Vp, m.vocab, m.seq_len, inv_n, st));
        PF_HIP(gemm_nt(m.dtype, t.logits, t.Et, t.d_ln, T, d, t.Vp, none, st));                 // dh = dlogits E
        float* dE = (float*)((char*)ge + t.emb32_off[0]);                                       // dE = dlogits^T h
        if (gemm_tn_acc_supported(m.dtype, t.logits, hf, t.Vp, d, T) && gemm_tn_acc_preferred(t.Vp, d, T)) {
          PF_HIP(gemm_tn_acc(m.dtype, t.logits, hf, dE, nullptr, t.Vp, d, T, st));
        } else {
          PF_HIP(transpose2d(m.dtype, t.logits, t.logitsT, T, t.Vp, st));                       // dlogits^T [Vp][T]
          PF_HIP(transpose2d(m.dtype, hf, t.tB, T, d, st));                                     // h^T [d][T]
          GemmEpilogue acc;
          acc.out_f32 = 1;
          acc.accumulate = 1;
          PF_HIP(gemm_nt(m.dtype, t.logitsT, t.tB, dE, t.Vp, d, T, acc, st));
        }
        // final LayerNorm backward (statistics recomputed from the checkpointed input)
        PF_HIP(layernorm_fwd(m.dtype, ck(mb, L), t.lnf_g_w, t.lnf_b_w, t.ln2, meanf, rstdf, T, d, m.eps, st));
        PF_HIP(layernorm_bwd(m.dtype, t.d_ln, ck(mb, L), t.lnf_g_w, meanf, rstdf, nullptr, t.G + mb * act,
                             (float*)((char*)ge + t.emb32_off[2]), (float*)((char*)ge + t.emb32_off[3]), t.ln_partial,
                             T, d, st));
        t.loss_count += 1;
      }
      return PF_OK;
    }
    default:
      return fail(PF_ERR_STATE, "training chunk: op %d is not a forward-type node", n.op);
  }
}

static int32_t optimizer_step(pf_ctx* c, hipStream_t st) {
  TrainState& t = *c->tr;
  const pf_adam& a = c->adam;
  const int64_t step = t.steps + 1;
  if (!t.dry) t.steps = step;
  const int32_t accum = (int32_t)t.mb_accum;
  for (int64_t l = 0; l < c->md.n_layers; ++l) {
    PF_HIP(adam_update(t.master[l], t.m[l], t.v[l], t.grad[l], t.blob32 / 4, a.lr, a.beta1, a.beta2, a.eps, step,
                       accum, st, t.dry));
    int32_t rc = recast_layer(c, (int32_t)l, st);
    if (rc != PF_OK) return rc;
  }
  if (t.Vp) {
    PF_HIP(adam_update(t.embM, t.embm, t.embv, t.embg, t.emb32 / 4, a.lr, a.beta1, a.beta2, a.eps, step, accum, st, t.dry));
    int32_t rc = recast_emb(c, st);
    if (rc != PF_OK) return rc;
  }
  t.mb_accum = 0;
  return PF_OK;
}

int32_t train_bwd_node(pf_ctx* c, const pf_node& n, int64_t replica, const void* grad_in, hipStream_t st) {
  TrainState& t = *c->tr;
  const pf_model_desc& m = c->md;
  const int64_t act = c->lay.act, T = c->lay.tokens, L = m.n_layers;
  const int32_t g = c->cfg.g;
  switch (n.op) {
    case PF_OP_LAYER_BWD:
      for (int32_t mb = 0; mb < g; ++mb) {
        char* G = t.G + mb * act;
        if (grad_in)
          PF_HIP(hipMemcpyAsync(G, (const char*)grad_in + mb * act, (size_t)act, hipMemcpyDeviceToDevice, st));
        int32_t rc = layer_backward(c, n.layer, t.ckpt + ((int64_t)mb * (L + 1) + n.layer) * act, G, st);
        if (rc != PF_OK) return rc;
      }
      return PF_OK;
    case PF_OP_OPT: {
      if (t.Vp) {
        const int32_t* ids = replica_ids(c, replica);
        if (!ids) return fail(PF_ERR_STATE, "training chunk: no input ring set (pf_ctx_set_io)");
        for (int32_t mb = 0; mb < g; ++mb)
          PF_HIP(embed_bwd(m.dtype, t.G + mb * act, ids + mb * T, (float*)((char*)t.embg + t.emb32_off[0]),
                           (float*)((char*)t.embg + t.emb32_off[1]), T, m.seq_len, m.d_model, m.vocab, st));
      }
      t.mb_accum += g;
      if (t.mb_accum >= c->adam.accum) return optimizer_step(c, st);
      return PF_OK;
    }
    default:
      return fail(PF_ERR_STATE, "training chunk: op %d is not a backward-type node", n.op);
  }
}

int32_t train_main_step(pf_ctx* c, int32_t instr, int32_t index, const void* io, hipStream_t st) {
  TrainState& t = *c->tr;
  const int64_t act = c->lay.act, L = c->md.n_layers;
  const int32_t slot = index % c->cfg.g;
  char* ck0 = t.ckpt + (int64_t)slot * (L + 1) * act;
  // A checkpoint slot serves one microbatch from its forward to its backward: a forward that lands on a slot still
  // in use would overwrite checkpoints a later backward reads (the context has fewer slots than microbatches in flight).
  if (instr == PF_INSTR_FWD && t.slot_live[slot])
    return fail(PF_ERR_STATE, "pf_main_stage_step: forward %d needs checkpoint slot %d, whose backward has not run "
                "(the context keeps g = %d microbatches in flight)", index, slot, c->cfg.g);
  if (instr == PF_INSTR_BWD && !t.slot_live[slot])
    return fail(PF_ERR_STATE, "pf_main_stage_step: backward %d has no forward in checkpoint slot %d", index, slot);
  t.slot_live[slot] = instr == PF_INSTR_FWD;
  if (instr == PF_INSTR_FWD) {
    PF_HIP(hipMemcpyAsync(ck0, io, (size_t)act, hipMemcpyDeviceToDevice, st));
    for (int64_t l = 0; l < L; ++l) {
      int32_t rc = layer_forward(c, t.Wk[l], ck0 + l * act, ck0 + (l + 1) * act, st);
      if (rc != PF_OK) return rc;
    }
    return PF_OK;
  }
  char* G = t.G + (int64_t)slot * act;
  PF_HIP(hipMemcpyAsync(G, io, (size_t)act, hipMemcpyDeviceToDevice, st));
  for (int64_t l = L - 1; l >= 0; --l) {
    int32_t rc = layer_backward(c, (int32_t)l, ck0 + l * act, G, st);
    if (rc != PF_OK) return rc;
  }
  return PF_OK;
}

int64_t train_opt_state_bytes(const pf_ctx* c) { return c->md.n_layers * 2 * c->tr->blob32; }

// Calls f(device address, offset in the string, length) for every contiguous piece of [off, off + len): a layer's
// two moment arrays lie next to each other in the arena, different layers do not.
template <class Fn>
static int32_t for_opt_state_pieces(pf_ctx* c, int64_t off, int64_t len, Fn&& f) {
  TrainState& t = *c->tr;
  const int64_t per_layer = 2 * t.blob32;
  if (off < 0 || len < 0 || off + len > train_opt_state_bytes(c)) return fail(PF_ERR_ARG, "optimizer state: range out of bounds");
  while (len > 0) {
    const int64_t l = off / per_layer, in_layer = off % per_layer;
    const int64_t n = std::min(len, per_layer - in_layer);
    if ((char*)t.v[l] != (char*)t.m[l] + t.blob32) return fail(PF_ERR_STATE, "optimizer state: moments are not adjacent");
    int32_t rc = f((char*)t.m[l] + in_layer, off, n);
    if (rc != PF_OK) return rc;
    off += n;
    len -= n;
  }
  return PF_OK;
}

int32_t train_opt_state_copy(pf_ctx* c, int64_t off, int64_t len, char* host, bool to_host, hipStream_t st) {
  return for_opt_state_pieces(c, off, len, [&](char* dev, int64_t o, int64_t n) -> int32_t {
    if (to_host) PF_HIP(hipMemcpyAsync(host + o, dev, (size_t)n, hipMemcpyDeviceToHost, st));
    else PF_HIP(hipMemcpyAsync(dev, host + o, (size_t)n, hipMemcpyHostToDevice, st));
    return PF_OK;
  });
}

int32_t train_opt_state_fill(pf_ctx* c, int64_t off, int64_t len, int32_t byte, hipStream_t st) {
  return for_opt_state_pieces(c, off, len, [&](char* dev, int64_t, int64_t n) -> int32_t {
    PF_HIP(hipMemsetAsync(dev, byte, (size_t)n, st));
    return PF_OK;
  });
}

int32_t train_main_opt(pf_ctx* c, int32_t microbatches, hipStream_t st) {
  c->tr->mb_accum = microbatches;
  return optimizer_step(c, st);
}

namespace {
struct ProfileSave { int64_t steps, loss_count; float loss; };
thread_local ProfileSave g_profile_save;
}  // namespace

int32_t train_profile_begin(pf_ctx* c, hipStream_t st) {
  TrainState& t = *c->tr;
  if (t.mb_accum != 0)
    return fail(PF_ERR_STATE, "pf_profile_chain: %lld microbatches are accumulated; profile a training context between "
                "optimizer steps", (long long)t.mb_accum);
  PF_HIP(hipStreamSynchronize(st));
  g_profile_save.steps = t.steps;
  g_profile_save.loss_count = t.loss_count;
  PF_HIP(hipMemcpy(&g_profile_save.loss, t.loss, sizeof(float), hipMemcpyDeviceToHost));
  t.dry = true;
  return PF_OK;
}

int32_t train_profile_end(pf_ctx* c, hipStream_t st) {
  TrainState& t = *c->tr;
  int32_t rc = PF_OK;
  if (t.mb_accum != 0) rc = optimizer_step(c, st);   // dry: clears the gradients the profiled nodes left behind
  t.dry = false;
  t.mb_accum = 0;
  t.steps = g_profile_save.steps;
  t.loss_count = g_profile_save.loss_count;
  if (rc != PF_OK) return rc;
  PF_HIP(hipStreamSynchronize(st));
  PF_HIP(hipMemcpy(t.loss, &g_profile_save.loss, sizeof(float), hipMemcpyHostToDevice));
  return PF_OK;
}

int32_t train_read_params(pf_ctx* c, int32_t what, int32_t layer, void* dst, int64_t dst_bytes, hipStream_t st) {
  TrainState& t = *c->tr;
  const void* src;
  int64_t n;
  if (layer >= 0) {
    if (layer >= c->md.n_layers) return fail(PF_ERR_ARG, "pf_ctx_read_params: layer out of range");
    src = what == 0 ? t.grad[layer] : what == 1 ? t.master[layer] : what == 2 ? t.m[layer] : t.v[layer];
    n = t.blob32;
  } else {
    if (!t.Vp) return fail(PF_ERR_STATE, "pf_ctx_read_params: the model has no embeddings");
    src = what == 0 ? t.embg : what == 1 ? t.embM : what == 2 ? t.embm : t.embv;
    n = t.emb32;
  }
  if (dst_bytes < n) return fail(PF_ERR_CAPACITY, "pf_ctx_read_params: %lld bytes needed", (long long)n);
  PF_HIP(hipMemcpyAsync(dst, src, (size_t)n, hipMemcpyDeviceToDevice, st));
  return PF_OK;
}

}  // namespace pf
