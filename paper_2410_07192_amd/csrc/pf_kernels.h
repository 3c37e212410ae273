// Launchers of the gfx950 kernels (internal).  Every launcher enqueues on `stream` and returns the
// launch status; none synchronises.  `dtype` is PF_DTYPE_F32 or PF_DTYPE_BF16 and names the storage
// type of activations and weights; accumulation and statistics are always fp32.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace pf {

// ---- GEMM  C[M,N] = op( X[M,K] * W[N,K]^T )  (both operands contiguous along K) -------------------
struct GemmEpilogue {
  const void* bias = nullptr;    // [N], model dtype: added to every row
  const void* resid = nullptr;   // [M,N], model dtype: added after the activation
  const void* dact_in = nullptr; // [M,N], model dtype: result multiplied by gelu'(dact_in)
  void* preact_out = nullptr;    // [M,N], model dtype: receives acc + bias before the activation
  int32_t gelu = 0;              // apply exact GELU after the bias
  int32_t accumulate = 0;        // fp32 output only: C += result
  int32_t out_f32 = 0;           // C is fp32 regardless of the model dtype
  float scale = 1.0f;            // result multiplied by this first
};
hipError_t gemm_nt(int32_t dtype, const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K,
                   const GemmEpilogue& ep, hipStream_t stream);

// C[M,N] (fp32) += A^T B with A [K,M] and B [K,N] row-major bf16 (weight gradient dW = dY^T X from the tensors as
// they lie in memory); colsum (fp32 [M], may be null): colsum[m] += sum over k of A[k][m].  Needs bf16, M and N
// multiples of 8, K a multiple of 64 and 16-byte aligned operands (gemm_tn_acc_supported); K may be split over
// workgroups, whose slices meet in C through fp32 atomics.
bool gemm_tn_acc_supported(int32_t dtype, const void* A, const void* B, int64_t M, int64_t N, int64_t K);
// whether it beats transposing both operands for the NT kernel (measured rates; large results favour the latter)
bool gemm_tn_acc_preferred(int64_t M, int64_t N, int64_t K);
hipError_t gemm_tn_acc(int32_t dtype, const void* A, const void* B, float* C, float* colsum, int64_t M, int64_t N,
                       int64_t K, hipStream_t stream);

// ---- LayerNorm ------------------------------------------------------------------------------------
// y = g * (x - mean) / sqrt(var + eps) + b per row of d elements.  mean_out / rstd_out (fp32 [rows])
// may be null.  warm / warm_bytes (optional): the kernel also reads that range and discards it, which leaves it
// in the memory-side cache; the callers name the weights of the GEMM that consumes y.
hipError_t layernorm_fwd(int32_t dtype, const void* x, const void* g, const void* b, void* y,
                         float* mean_out, float* rstd_out, int64_t rows, int32_t d, float eps,
                         hipStream_t stream, const void* warm = nullptr, int64_t warm_bytes = 0);

// ---- attention ------------------------------------------------------------------------------------
// qkv: [B*S, 3*d] rows = tokens, columns = Q | K | V blocks, head i at columns i*dh.. of each block.
// out: [B*S, d].  lse (fp32 [B, h, S], may be null) receives log-sum-exp of the scaled scores.
hipError_t attention_fwd(int32_t dtype, const void* qkv, void* out, float* lse, int32_t B, int32_t S,
                         int32_t h, int32_t dh, int32_t causal, hipStream_t stream);

// ---- embedding ------------------------------------------------------------------------------------
// x[t] = tok[ids[t]] + pos[t mod S];  ids outside [0, V) produce rows of zeros plus the position.
hipError_t embed_fwd(int32_t dtype, const int32_t* ids, const void* tok, const void* pos, void* x,
                     int64_t tokens, int32_t S, int32_t d, int32_t V, hipStream_t stream);

// ---- training-only kernels -----------------------------------------------------------------------------
// out[c][r] = in[r][c]
hipError_t transpose2d(int32_t dtype, const void* in, void* out, int64_t R, int64_t C, hipStream_t stream);
// acc[n] += sum over rows of x[row][n]   (fp32 atomics)
hipError_t colsum_add(int32_t dtype, const void* x, float* acc, int64_t rows, int64_t N, hipStream_t stream);
// both at once: out[c][r] = in[r][c] and acc[c] += sum over r of in[r][c]
hipError_t transpose2d_colsum(int32_t dtype, const void* in, void* out, float* acc, int64_t R, int64_t C,
                              hipStream_t stream);
// LayerNorm backward: dx = LN'(dy) (+ resid), dg += sum dy*xhat, db += sum dy.  dx may alias resid or dy.
// partial: fp32 scratch of max_blocks * 2 * d elements (one partial dg | db row per workgroup; at most
// LN_BWD_MAX_BLOCKS * 4 workgroups).
constexpr int64_t LN_BWD_MAX_BLOCKS = 128;
hipError_t layernorm_bwd(int32_t dtype, const void* dy, const void* x, const void* g, const float* mean,
                         const float* rstd, const void* resid, void* dx, float* dg, float* db, float* partial,
                         int64_t rows, int32_t d, hipStream_t stream, int64_t max_blocks = LN_BWD_MAX_BLOCKS * 4);
// Attention backward from the saved log-sum-exp.  dqkv: [B*S][3*d] like qkv; Dsum: fp32 [B][h][S] scratch.
hipError_t attention_bwd(int32_t dtype, const void* qkv, const void* o, const void* dout, const float* lse,
                         float* Dsum, void* dqkv, int32_t B, int32_t S, int32_t h, int32_t dh, int32_t causal,
                         hipStream_t stream);
// bf16, d_head 64 / 128: MFMA version (called by attention_bwd)
hipError_t attention_bwd_mfma(const void* qkv, const void* o, const void* dout, const float* lse, float* Dsum,
                              void* dqkv, int32_t B, int32_t S, int32_t h, int32_t dh, int32_t causal,
                              hipStream_t stream);
// In place on logits [tokens][pitch]: (softmax - onehot(next token)) * inv_n; loss_sum += -log p[target].
hipError_t ce_loss_inplace(int32_t dtype, void* logits, const int32_t* ids, float* loss_sum, int64_t tokens,
                           int64_t pitch, int32_t V, int32_t S, float inv_n, hipStream_t stream);
hipError_t embed_bwd(int32_t dtype, const void* dx, const int32_t* ids, float* dtok, float* dpos, int64_t tokens,
                     int32_t S, int32_t d, int32_t V, hipStream_t stream);
// Adam with bias correction on fp32 arrays; g holds the sum over `accum` microbatches and is cleared.
// dry: the same kernel with a zero step and unit decay factors, so theta, m and v keep their values (for profiling).
hipError_t adam_update(float* theta, float* m, float* v, float* g, int64_t n, float lr, float b1, float b2, float eps,
                       int64_t step, int32_t accum, hipStream_t stream, bool dry = false);
// fp32 [R][C] -> dst [R][C] in `dtype` and, if dst_t is not null, dst_t [C][R]
hipError_t cast_from_f32(int32_t dtype, const float* src, void* dst, void* dst_t, int64_t R, int64_t C,
                         hipStream_t stream);
hipError_t widen_to_f32(int32_t dtype, const void* src, float* dst, int64_t n, hipStream_t stream);

}  // namespace pf
