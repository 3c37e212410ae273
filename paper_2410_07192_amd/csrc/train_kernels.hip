// Kernels that only training fill jobs (and the emulated main-job stage) need: transposes for the
// weight-gradient GEMMs, bias-gradient column sums, LayerNorm backward, attention backward, the
// tied-head cross-entropy, embedding backward, Adam and the re-cast of master weights.
//
// All of these are HBM-bound (or, for the attention backward, plain-ALU bound in this first
// version): 16-byte accesses where the layout allows, fp32 arithmetic, fp32 atomics for the
// reductions over tokens (bias, LayerNorm scale/shift and embedding gradients), which makes those
// sums order-dependent in the last bits.
#include <mutex>

#include "pf_internal.h"
#include "pf_kernels.h"
#include "pf_device.h"

namespace pf {
namespace {

// ---- transpose: out[c][r] = in[r][c] ---------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, T* __restrict__ out, int64_t R,
                                                        int64_t Cn) {
  __shared__ T tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = ty * 16 + i;
    if (r0 + r < R && c0 + tx < Cn) tile[r][tx] = in[(r0 + r) * Cn + c0 + tx];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = ty * 16 + i;
    if (c0 + c < Cn && r0 + tx < R) out[(c0 + c) * R + r0 + tx] = tile[tx][c];
  }
}

// bf16 with R and Cn multiples of 8 and 16-byte aligned pointers: 64x64 tiles, 16-byte global accesses on both
// sides (a row of the tile is one 128-byte line), the transposition itself happens in LDS (dword writes,
// 2-byte reads at a pitch of 33 dwords, which spreads the eight row groups a wave reads over distinct banks).
// COLSUM: acc[c] += sum over r of in[r][c] on the way (fp32 atomics, one per column and 64-row tile): the
// bias gradient of a linear layer is the column sum of the very tensor whose transpose feeds its weight gradient.
template <bool COLSUM>
__global__ __launch_bounds__(256) void transpose_bf16_vec_kernel(const uint16_t* __restrict__ in,
                                                                 uint16_t* __restrict__ out, int64_t R, int64_t Cn,
                                                                 float* __restrict__ acc) {
  constexpr int PITCH = 66;   // elements
  __shared__ uint32_t tile32[64 * PITCH / 2];
  const uint16_t* tile = reinterpret_cast<const uint16_t*>(tile32);
  const int t = threadIdx.x;
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int q = t + k * 256, r = q >> 3, cc = (q & 7) * 8;
    if (r0 + r < R && c0 + cc < Cn) {
      const uint4 v = *reinterpret_cast<const uint4*>(in + (r0 + r) * Cn + c0 + cc);
      uint32_t* dst = tile32 + (r * PITCH + cc) / 2;
      dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int q = t + k * 256, c = q >> 3, rr = (q & 7) * 8;
    float sum = 0.f;
    if (c0 + c < Cn && r0 + rr < R) {
      uint32_t w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        w[j] = (uint32_t)tile[(rr + 2 * j) * PITCH + c] | ((uint32_t)tile[(rr + 2 * j + 1) * PITCH + c] << 16);
        if constexpr (COLSUM) sum += __uint_as_float(w[j] << 16) + __uint_as_float(w[j] & 0xffff0000u);
      }
      *reinterpret_cast<uint4*>(out + (c0 + c) * R + r0 + rr) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if constexpr (COLSUM) {   // the eight lanes that share column c hold its eight row groups
      sum += __shfl_xor(sum, 1, 64);
      sum += __shfl_xor(sum, 2, 64);
      sum += __shfl_xor(sum, 4, 64);
      if ((t & 7) == 0 && c0 + c < Cn) unsafeAtomicAdd(acc + c0 + c, sum);
    }
  }
}

// ---- column sums: acc[n] += sum_t x[t][n] -----------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ x, float* __restrict__ acc, int64_t rows,
                                                     int64_t N, int32_t rows_per_block) {
  const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  const int64_t r1 = (r0 + rows_per_block < rows) ? r0 + rows_per_block : rows;
  float s = 0.f;
  for (int64_t r = r0; r < r1; ++r) s += to_f32(x[r * N + n]);
  unsafeAtomicAdd(acc + n, s);
}

// bf16, N a multiple of 8, 16-byte aligned rows: a block covers 1024 columns (128 threads x 8) with two row
// lanes, 16-byte loads, four rows in flight per thread; the two lanes meet in LDS before the atomics.
__global__ __launch_bounds__(256) void colsum_bf16_vec_kernel(const bf16_t* __restrict__ x, float* __restrict__ acc,
                                                              int64_t rows, int64_t N, int32_t rows_per_block) {
  __shared__ float part[128][8];
  const int cg = threadIdx.x & 127, rl = threadIdx.x >> 7;
  const int64_t c0 = (int64_t)blockIdx.x * 1024 + cg * 8;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  const int64_t r1 = (r0 + rows_per_block < rows) ? r0 + rows_per_block : rows;
  float s[8] = {};
  if (c0 < N) {
    int64_t r = r0 + rl;
    for (; r + 6 < r1; r += 8) {
      float v[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) load8(x + (r + 2 * u) * N + c0, v[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 8; ++j) s[j] += v[u][j];
    }
    for (; r < r1; r += 2) {
      float v[8];
      load8(x + r * N + c0, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) s[j] += v[j];
    }
  }
  if (rl == 1) {
#pragma unroll
    for (int j = 0; j < 8; ++j) part[cg][j] = s[j];
  }
  __syncthreads();
  if (rl == 0 && c0 < N) {
#pragma unroll
    for (int j = 0; j < 8; ++j) unsafeAtomicAdd(acc + c0 + j, s[j] + part[cg][j]);
  }
}

// ---- LayerNorm backward -----------------------------------------------------------------------------
// dx = rstd * (g*dy - mean(g*dy) - xhat * mean(g*dy*xhat)) [+ resid];  dg += sum dy*xhat;  db += sum dy.
// One workgroup of NW waves per row, rows strided over the grid; a thread keeps ITER groups of 8 columns
// and its partial dg/db in registers; the next row's x and dy are fetched before this row's two sums are
// reduced (wave shuffle, then through LDS across the waves: one barrier per row, the LDS slots alternate).
// Each workgroup writes one partial row to `partial` ([workgroups][2][d]) and a second kernel sums the rows
// in a fixed order (deterministic) into dg / db.
template <typename T, int NW, int ITER, bool HAS_RESID>
__global__ __launch_bounds__(64 * NW) void layernorm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                const T* __restrict__ g, const float* __restrict__ mean,
                                                                const float* __restrict__ rstd, const T* resid, T* dx,
                                                                float* __restrict__ partial, int64_t rows, int32_t d) {
  typedef typename Raw8<T>::type raw_t;
  __shared__ float red[2][NW][2];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  float pg[ITER][8], pb[ITER][8], gg[ITER][8];
  int cc[ITER];   // column of group i, or 0 for a group past the end (loaded like the others, never used)
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int c = (i * 64 * NW + t) * 8;
    cc[i] = c < d ? c : 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) pg[i][j] = pb[i][j] = 0.f;
    load8(g + cc[i], gg[i]);
  }
  // the next row's x and dy stay raw in registers while this row is reduced: converting them on arrival would
  // put the wait for the load right behind it
  raw_t xr[ITER], dr[ITER];
  auto fetch = [&](int64_t r) {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      xr[i] = *(const raw_t*)(x + r * d + cc[i]);
      dr[i] = *(const raw_t*)(dy + r * d + cc[i]);
    }
  };
  int64_t row = blockIdx.x;
  if (row < rows) fetch(row);
  int par = 0;
  for (; row < rows; row += gridDim.x) {
    const float mu = mean[row], rs = rstd[row];
    float xh[ITER][8], dv[ITER][8];
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      unpack8(xr[i], xh[i]);
      unpack8(dr[i], dv[i]);
    }
    // requested in the order they are needed: the residual (at the end of this row), then the next row
    raw_t rres[HAS_RESID ? ITER : 1];
    if constexpr (HAS_RESID) {
#pragma unroll
      for (int i = 0; i < ITER; ++i) rres[i] = *(const raw_t*)(resid + row * d + cc[i]);
    }
    {
      const int64_t nxt = row + gridDim.x;
      fetch(nxt < rows ? nxt : row);   // the last row is asked for once more rather than branched around
    }
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int c = (i * 64 * NW + t) * 8;
      if (c < d) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          xh[i][j] = (xh[i][j] - mu) * rs;
          pg[i][j] += dv[i][j] * xh[i][j];
          pb[i][j] += dv[i][j];
          dv[i][j] *= gg[i][j];
          s1 += dv[i][j];
          s2 += dv[i][j] * xh[i][j];
        }
      }
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if constexpr (NW > 1) {
      if (lane == 0) {
        red[par][wv][0] = s1;
        red[par][wv][1] = s2;
      }
      __syncthreads();
      s1 = s2 = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        s1 += red[par][w][0];
        s2 += red[par][w][1];
      }
      par ^= 1;
    }
    s1 /= (float)d;
    s2 /= (float)d;
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int c = (i * 64 * NW + t) * 8;
      float rr[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if constexpr (HAS_RESID) unpack8(rres[i], rr);
      if (c < d) {
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = (dv[i][j] - s1 - xh[i][j] * s2) * rs + rr[j];
        store8(dx + row * d + c, o);
      }
    }
  }
  float* pr = partial + (int64_t)blockIdx.x * 2 * (int64_t)d;
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int c = (i * 64 * NW + t) * 8;
    if (c < d) {
      store8(pr + c, pg[i]);
      store8(pr + d + c, pb[i]);
    }
  }
}

// dg[c] / db[c] += sum over rows of partial[row][c]  (partial is [n_rows][2*d]).  16 columns per workgroup
// (64 bytes of a row per 16 lanes), 64 row lanes per column, fixed summation order (deterministic).
__global__ __launch_bounds__(1024) void reduce_rows_add_kernel(const float* __restrict__ partial, float* __restrict__ dg,
                                                               float* __restrict__ db, int32_t n_rows, int32_t d) {
  __shared__ float red[64][17];
  const int cx = threadIdx.x & 15, ry = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cx;
  const int cl = c < 2 * d ? c : 0;   // a column past the end reads column 0 and is dropped below
  float s = 0.f;
  // eight rows per round, all requested before the first is added (a row past the end repeats the last one with
  // weight 0): one memory round trip for the 512 rows the LayerNorm kernel writes at most
  for (int r0 = ry; r0 < n_rows; r0 += 8 * 64) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int r = r0 + 64 * k;
      v[k] = partial[(int64_t)(r < n_rows ? r : n_rows - 1) * 2 * d + cl];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) s += (r0 + 64 * k < n_rows) ? v[k] : 0.f;
  }
  red[ry][cx] = s;
  __syncthreads();
  // fixed order: 16 lanes per column add four rows each, then lane 0 adds the sixteen
  const int col = threadIdx.x >> 4, part = threadIdx.x & 15;   // threads 0..255: column col, rows 4 part .. 4 part + 3
  float t = 0.f;
  if (threadIdx.x < 256) t = (red[4 * part][col] + red[4 * part + 1][col]) + (red[4 * part + 2][col] + red[4 * part + 3][col]);
  __syncthreads();
  if (threadIdx.x < 256) red[part][col] = t;
  __syncthreads();
  if (threadIdx.x < 16) {
    const int cc = blockIdx.x * 16 + threadIdx.x;
    float u = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) u += red[k][threadIdx.x];
    if (cc < 2 * d) {
      if (cc < d) dg[cc] += u;
      else db[cc - d] += u;
    }
  }
}

// ---- attention backward, one thread per row ----------------------------------------------------------
// dQ pass: thread = query.  Also writes D[q] = sum_j dO[q][j] * O[q][j].
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_bwd_dq_kernel(const T* __restrict__ qkv, const T* __restrict__ o,
                                                         const T* __restrict__ dout, const float* __restrict__ lse,
                                                         float* __restrict__ Dsum, T* __restrict__ dqkv, int32_t S,
                                                         int32_t h, int32_t causal, float scale) {
  constexpr int KT = 32;
  __shared__ float sK[KT][DH];
  __shared__ float sV[KT][DH];
  const int tid = threadIdx.x, b = blockIdx.z, hd = blockIdx.y;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * S * rs + hd * DH;
  const int q_row = blockIdx.x * 64 + tid;
  const bool live = q_row < S;
  float q[DH], dO[DH], dq[DH];
  float Dq = 0.f, L = 0.f;
#pragma unroll
  for (int j = 0; j < DH; ++j) {
    q[j] = live ? to_f32(base[(int64_t)q_row * rs + j]) : 0.f;
    dO[j] = live ? to_f32(dout[((int64_t)b * S + q_row) * d + hd * DH + j]) : 0.f;
    const float ov = live ? to_f32(o[((int64_t)b * S + q_row) * d + hd * DH + j]) : 0.f;
    Dq += dO[j] * ov;
    dq[j] = 0.f;
  }
  if (live) {
    L = lse[((int64_t)b * h + hd) * S + q_row];
    Dsum[((int64_t)b * h + hd) * S + q_row] = Dq;
  }
  int k_end = S;
  if (causal) {
    const int last_q = (blockIdx.x * 64 + 63 < S - 1) ? blockIdx.x * 64 + 63 : S - 1;
    k_end = last_q + 1;
  }
  for (int k0 = 0; k0 < k_end; k0 += KT) {
    __syncthreads();
    for (int i = tid; i < KT * DH; i += 64) {
      const int r = i / DH, c = i % DH;
      const bool ok = k0 + r < S;
      sK[r][c] = ok ? to_f32(base[(int64_t)(k0 + r) * rs + d + c]) : 0.f;
      sV[r][c] = ok ? to_f32(base[(int64_t)(k0 + r) * rs + 2 * d + c]) : 0.f;
    }
    __syncthreads();
    if (!live) continue;
    for (int r = 0; r < KT; ++r) {
      const int key = k0 + r;
      if (key >= S || (causal && key > q_row)) continue;
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int j = 0; j < DH; ++j) {
        s = fmaf(q[j], sK[r][j], s);
        dp = fmaf(dO[j], sV[r][j], dp);
      }
      const float p = __expf(s * scale - L);
      const float ds = p * (dp - Dq) * scale;
#pragma unroll
      for (int j = 0; j < DH; ++j) dq[j] = fmaf(ds, sK[r][j], dq[j]);
    }
  }
  if (live) {
    T* out = dqkv + ((int64_t)b * S + q_row) * rs + hd * DH;
#pragma unroll
    for (int j = 0; j < DH; ++j) out[j] = from_f32<T>(dq[j]);
  }
}

// dK / dV pass: thread = key.
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_bwd_dkv_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                          const float* __restrict__ lse,
                                                          const float* __restrict__ Dsum, T* __restrict__ dqkv,
                                                          int32_t S, int32_t h, int32_t causal, float scale) {
  constexpr int QT = 32;
  __shared__ float sQ[QT][DH];
  __shared__ float sdO[QT][DH];
  __shared__ float sL[QT], sD[QT];
  const int tid = threadIdx.x, b = blockIdx.z, hd = blockIdx.y;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * S * rs + hd * DH;
  const int k_row = blockIdx.x * 64 + tid;
  const bool live = k_row < S;
  float k[DH], v[DH], dk[DH], dv[DH];
#pragma unroll
  for (int j = 0; j < DH; ++j) {
    k[j] = live ? to_f32(base[(int64_t)k_row * rs + d + j]) : 0.f;
    v[j] = live ? to_f32(base[(int64_t)k_row * rs + 2 * d + j]) : 0.f;
    dk[j] = dv[j] = 0.f;
  }
  const int q_begin = causal ? (blockIdx.x * 64) / QT * QT : 0;   // earlier queries never see these keys
  for (int q0 = q_begin; q0 < S; q0 += QT) {
    __syncthreads();
    for (int i = tid; i < QT * DH; i += 64) {
      const int r = i / DH, c = i % DH;
      const bool ok = q0 + r < S;
      sQ[r][c] = ok ? to_f32(base[(int64_t)(q0 + r) * rs + c]) : 0.f;
      sdO[r][c] = ok ? to_f32(dout[((int64_t)b * S + q0 + r) * d + hd * DH + c]) : 0.f;
    }
    if (tid < QT) {
      const bool ok = q0 + tid < S;
      sL[tid] = ok ? lse[((int64_t)b * h + hd) * S + q0 + tid] : 0.f;
      sD[tid] = ok ? Dsum[((int64_t)b * h + hd) * S + q0 + tid] : 0.f;
    }
    __syncthreads();
    if (!live) continue;
    for (int r = 0; r < QT; ++r) {
      const int qi = q0 + r;
      if (qi >= S || (causal && k_row > qi)) continue;
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int j = 0; j < DH; ++j) {
        s = fmaf(sQ[r][j], k[j], s);
        dp = fmaf(sdO[r][j], v[j], dp);
      }
      const float p = __expf(s * scale - sL[r]);
      const float ds = p * (dp - sD[r]) * scale;
#pragma unroll
      for (int j = 0; j < DH; ++j) {
        dv[j] = fmaf(p, sdO[r][j], dv[j]);
        dk[j] = fmaf(ds, sQ[r][j], dk[j]);
      }
    }
  }
  if (live) {
    T* out = dqkv + ((int64_t)b * S + k_row) * rs + hd * DH;
#pragma unroll
    for (int j = 0; j < DH; ++j) {
      out[d + j] = from_f32<T>(dk[j]);
      out[2 * d + j] = from_f32<T>(dv[j]);
    }
  }
}

// ---- tied-head cross-entropy -------------------------------------------------------------------------
// One workgroup per token row.  logits: [T][pitch] (columns >= V are padding).  Row t predicts
// ids[t+1] unless t is the last position of its sequence.  In place: logits <- (softmax - onehot) *
// inv_n (zeros for rows without target and for padding); loss_sum += -log softmax[target].
template <typename T>
__global__ __launch_bounds__(256) void ce_loss_kernel(T* __restrict__ logits, const int32_t* __restrict__ ids,
                                                      float* __restrict__ loss_sum, int64_t pitch, int32_t V, int32_t S,
                                                      float inv_n) {
  __shared__ float red[4];
  const int64_t t = blockIdx.x;
  T* row = logits + t * pitch;
  const int tid = threadIdx.x;
  const bool has_target = (t % S) != S - 1;
  if (!has_target) {
    for (int64_t c = tid; c < pitch; c += 256) row[c] = from_f32<T>(0.f);
    return;
  }
  float mx = -INFINITY;
  for (int c = tid; c < V; c += 256) mx = fmaxf(mx, to_f32(row[c]));
  mx = wave_max(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float se = 0.f;
  for (int c = tid; c < V; c += 256) se += __expf(to_f32(row[c]) - mx);
  se = wave_sum(se);
  if ((tid & 63) == 0) red[tid >> 6] = se;
  __syncthreads();
  se = red[0] + red[1] + red[2] + red[3];
  const int32_t tgt = ids[t + 1];
  const float inv = 1.f / se;
  if (tid == 0 && tgt >= 0 && tgt < V) unsafeAtomicAdd(loss_sum, (mx + __logf(se)) - to_f32(row[tgt]));
  __syncthreads();   // the target logit is read before anyone overwrites the row
  for (int64_t c = tid; c < pitch; c += 256) {
    float gval = 0.f;
    if (c < V) gval = (__expf(to_f32(row[c]) - mx) * inv - (c == tgt ? 1.f : 0.f)) * inv_n;
    row[c] = from_f32<T>(gval);
  }
}

// bf16 rows with a pitch that is a multiple of 8: 16-byte accesses, running (max, sum) in one pass over the row,
// then one pass that rewrites it (two reads and one write of the logits instead of three reads and one write).
__global__ __launch_bounds__(256) void ce_loss_bf16_vec_kernel(bf16_t* __restrict__ logits, const int32_t* __restrict__ ids,
                                                               float* __restrict__ loss_sum, int64_t pitch, int32_t V,
                                                               int32_t S, float inv_n) {
  __shared__ float red_m[4], red_s[4];
  const int64_t t = blockIdx.x;
  bf16_t* row = logits + t * pitch;
  const int tid = threadIdx.x;
  const int chunks = (int)(pitch / 8);
  if ((t % S) == S - 1) {   // no target: zero gradient
    for (int c = tid; c < chunks; c += 256) *(uint4*)(row + c * 8) = make_uint4(0, 0, 0, 0);
    return;
  }
  float mx = -INFINITY, se = 0.f;
  for (int c = tid; c < chunks; c += 256) {
    float v[8];
    load8(row + c * 8, v);
    float cm = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (c * 8 + j < V) cm = fmaxf(cm, v[j]);
    if (cm > mx) {
      se *= __expf(mx - cm);   // mx = -inf: se is 0 and stays 0
      mx = cm;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (c * 8 + j < V) se += __expf(v[j] - mx);
  }
  // combine the lanes: (max, sum) pairs
  const float wm = wave_max(mx);
  se = wave_sum(mx == -INFINITY ? 0.f : se * __expf(mx - wm));
  if ((tid & 63) == 0) {
    red_m[tid >> 6] = wm;
    red_s[tid >> 6] = se;
  }
  const int32_t tgt = ids[t + 1];
  const float tgt_logit = (tgt >= 0 && tgt < V) ? to_f32(row[tgt]) : 0.f;   // read before the row is rewritten
  __syncthreads();
  const float m = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));
  float sum = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) sum += red_s[w] * __expf(red_m[w] - m);
  const float inv = 1.f / sum;
  if (tid == 0 && tgt >= 0 && tgt < V) unsafeAtomicAdd(loss_sum, (m + __logf(sum)) - tgt_logit);
  for (int c = tid; c < chunks; c += 256) {
    float v[8];
    load8(row + c * 8, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int col = c * 8 + j;
      v[j] = (col < V) ? (__expf(v[j] - m) * inv - (col == tgt ? 1.f : 0.f)) * inv_n : 0.f;
    }
    store8(row + c * 8, v);
  }
}

// ---- embedding backward: dtok[ids[t]] += dx[t], dpos[t mod S] += dx[t] --------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(const T* __restrict__ dx, const int32_t* __restrict__ ids,
                                                        float* __restrict__ dtok, float* __restrict__ dpos,
                                                        int64_t tokens, int32_t S, int32_t d, int32_t V) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= tokens) return;
  const int32_t id = ids[t];
  const bool ok = id >= 0 && id < V;
  // one column per lane and instruction: an atomic instruction then covers 256 consecutive bytes of the row
  // (eight columns per lane would spread it over sixteen cache lines)
  float* trow = dtok + (int64_t)(ok ? id : 0) * d;
  float* prow = dpos + (t % S) * (int64_t)d;
  for (int c = lane; c < d; c += 64) {
    const float v = to_f32(dx[t * d + c]);
    if (ok) unsafeAtomicAdd(trow + c, v);
    unsafeAtomicAdd(prow + c, v);
  }
}

// ---- Adam ------------------------------------------------------------------------------------------------
// g is the SUM over `accum` microbatches; the step uses g/accum and clears g.
__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ theta, float* __restrict__ m, float* __restrict__ v,
                                                   float* __restrict__ g, int64_t n, float lr, float b1, float b2,
                                                   float eps, float bc1, float bc2, float inv_accum) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float gr = g[i] * inv_accum;
  const float mi = b1 * m[i] + (1.f - b1) * gr;
  const float vi = b2 * v[i] + (1.f - b2) * gr * gr;
  m[i] = mi;
  v[i] = vi;
  theta[i] -= lr * (mi / bc1) / (sqrtf(vi / bc2) + eps);
  g[i] = 0.f;
}

// master (fp32) -> working copy in the model dtype; for a matrix [R][C] also the transposed copy [C][R]
template <typename T>
__global__ __launch_bounds__(256) void cast_kernel(const float* __restrict__ src, T* __restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = from_f32<T>(src[i]);
}
template <typename T>
__global__ __launch_bounds__(256) void cast_transpose_kernel(const float* __restrict__ src, T* __restrict__ dst,
                                                             T* __restrict__ dst_t, int64_t R, int64_t Cn) {
  __shared__ float tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = ty * 16 + i;
    if (r0 + r < R && c0 + tx < Cn) {
      const float val = src[(r0 + r) * Cn + c0 + tx];
      tile[r][tx] = val;
      dst[(r0 + r) * Cn + c0 + tx] = from_f32<T>(val);
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = ty * 16 + i;
    if (c0 + c < Cn && r0 + tx < R) dst_t[(c0 + c) * R + r0 + tx] = from_f32<T>(tile[tx][c]);
  }
}
template <typename T>
__global__ __launch_bounds__(256) void widen_kernel(const T* __restrict__ src, float* __restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = to_f32(src[i]);
}

#define PF_BY_DTYPE(dtype, CALL_BF16, CALL_F32) \
  do {                                          \
    if ((dtype) == PF_DTYPE_BF16_) { CALL_BF16; } else { CALL_F32; } \
  } while (0)

}  // namespace

hipError_t transpose2d(int32_t dtype, const void* in, void* out, int64_t R, int64_t Cn, hipStream_t st) {
  if (R <= 0 || Cn <= 0) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((Cn + 63) / 64), (unsigned)((R + 63) / 64));
  if (grid.y > 65535) return hipErrorInvalidValue;
  if (dtype == PF_DTYPE_BF16_ && R % 8 == 0 && Cn % 8 == 0 && (((uintptr_t)in | (uintptr_t)out) & 15) == 0) {
    hipLaunchKernelGGL(transpose_bf16_vec_kernel<false>, grid, dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out, R,
                       Cn, (float*)nullptr);
    return hipGetLastError();
  }
  PF_BY_DTYPE(dtype,
              hipLaunchKernelGGL(transpose_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)in, (bf16_t*)out, R, Cn),
              hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, st, (const float*)in, (float*)out, R, Cn));
  return hipGetLastError();
}

hipError_t colsum_add(int32_t dtype, const void* x, float* acc, int64_t rows, int64_t N, hipStream_t st) {
  if (rows <= 0 || N <= 0) return hipErrorInvalidValue;
  if (dtype == PF_DTYPE_BF16_ && N % 8 == 0 && ((uintptr_t)x & 15) == 0) {
    const int32_t rpb = 128;
    const dim3 grid((unsigned)((N + 1023) / 1024), (unsigned)((rows + rpb - 1) / rpb));
    if (grid.y > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(colsum_bf16_vec_kernel, grid, dim3(256), 0, st, (const bf16_t*)x, acc, rows, N, rpb);
    return hipGetLastError();
  }
  const int32_t rpb = 128;
  const dim3 grid((unsigned)((N + 255) / 256), (unsigned)((rows + rpb - 1) / rpb));
  if (grid.y > 65535) return hipErrorInvalidValue;
  PF_BY_DTYPE(dtype,
              hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)x, acc, rows, N, rpb),
              hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)x, acc, rows, N, rpb));
  return hipGetLastError();
}

hipError_t transpose2d_colsum(int32_t dtype, const void* in, void* out, float* acc, int64_t R, int64_t Cn,
                              hipStream_t st) {
  if (R <= 0 || Cn <= 0 || !acc) return hipErrorInvalidValue;
  if (dtype == PF_DTYPE_BF16_ && R % 8 == 0 && Cn % 8 == 0 && (((uintptr_t)in | (uintptr_t)out) & 15) == 0) {
    const dim3 grid((unsigned)((Cn + 63) / 64), (unsigned)((R + 63) / 64));
    if (grid.y > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(transpose_bf16_vec_kernel<true>, grid, dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out, R, Cn,
                       acc);
    return hipGetLastError();
  }
  hipError_t e = transpose2d(dtype, in, out, R, Cn, st);
  return e != hipSuccess ? e : colsum_add(dtype, in, acc, R, Cn, st);
}

template <typename T>
static hipError_t launch_ln_bwd(const void* dy, const void* x, const void* g, const float* mean, const float* rstd,
                                const void* resid, void* dx, float* dg, float* db, float* partial, int64_t rows,
                                int32_t d, hipStream_t st, int64_t max_blocks) {
  int64_t blocks = rows;
  if (blocks > max_blocks) blocks = max_blocks;   // rows of `partial`
  const dim3 grid((unsigned)blocks);
#define PF_LNB(NW, I)                                                                                            \
  do {                                                                                                           \
    if (resid)                                                                                                   \
      hipLaunchKernelGGL((layernorm_bwd_kernel<T, NW, I, true>), grid, dim3(64 * NW), 0, st, (const T*)dy,       \
                         (const T*)x, (const T*)g, mean, rstd, (const T*)resid, (T*)dx, partial, rows, d);       \
    else                                                                                                         \
      hipLaunchKernelGGL((layernorm_bwd_kernel<T, NW, I, false>), grid, dim3(64 * NW), 0, st, (const T*)dy,      \
                         (const T*)x, (const T*)g, mean, rstd, (const T*)resid, (T*)dx, partial, rows, d);       \
  } while (0)
  if (d <= 512) PF_LNB(1, 1);
  else if (d <= 1024) PF_LNB(2, 1);
  else if (d <= 2048) PF_LNB(4, 1);
  else if (d <= 4096) PF_LNB(4, 2);
  else if (d <= 8192) PF_LNB(4, 4);
  else return hipErrorInvalidValue;
#undef PF_LNB
  hipLaunchKernelGGL(reduce_rows_add_kernel, dim3((unsigned)((2 * d + 15) / 16)), dim3(1024), 0, st, partial, dg, db,
                     (int32_t)blocks, d);
  return hipGetLastError();
}

hipError_t layernorm_bwd(int32_t dtype, const void* dy, const void* x, const void* g, const float* mean,
                         const float* rstd, const void* resid, void* dx, float* dg, float* db, float* partial,
                         int64_t rows, int32_t d, hipStream_t st, int64_t max_blocks) {
  if (rows <= 0 || d <= 0 || d % 8 != 0 || d > 8192 || !partial || max_blocks < 1 || max_blocks > LN_BWD_MAX_BLOCKS * 4)
    return hipErrorInvalidValue;
  if (dtype == PF_DTYPE_BF16_)
    return launch_ln_bwd<bf16_t>(dy, x, g, mean, rstd, resid, dx, dg, db, partial, rows, d, st, max_blocks);
  return launch_ln_bwd<float>(dy, x, g, mean, rstd, resid, dx, dg, db, partial, rows, d, st, max_blocks);
}

template <typename T>
static hipError_t launch_attn_bwd(const void* qkv, const void* o, const void* dout, const float* lse, float* Dsum,
                                  void* dqkv, int32_t B, int32_t S, int32_t h, int32_t dh, int32_t causal,
                                  hipStream_t st) {
  const dim3 grid((unsigned)((S + 63) / 64), (unsigned)h, (unsigned)B), block(64);
  const float scale = 1.0f / sqrtf((float)dh);
#define PF_AB(D)                                                                                               \
  do {                                                                                                         \
    hipLaunchKernelGGL((attn_bwd_dq_kernel<T, D>), grid, block, 0, st, (const T*)qkv, (const T*)o, (const T*)dout, \
                       lse, Dsum, (T*)dqkv, S, h, causal, scale);                                              \
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<T, D>), grid, block, 0, st, (const T*)qkv, (const T*)dout, lse, Dsum, \
                       (T*)dqkv, S, h, causal, scale);                                                         \
  } while (0)
  switch (dh) {
    case 8: PF_AB(8); break;
    case 16: PF_AB(16); break;
    case 32: PF_AB(32); break;
    case 64: PF_AB(64); break;
    case 128: PF_AB(128); break;
    default: return hipErrorInvalidValue;
  }
#undef PF_AB
  return hipGetLastError();
}

hipError_t attention_bwd(int32_t dtype, const void* qkv, const void* o, const void* dout, const float* lse,
                         float* Dsum, void* dqkv, int32_t B, int32_t S, int32_t h, int32_t dh, int32_t causal,
                         hipStream_t st) {
  if (B <= 0 || S <= 0 || h <= 0 || B > 65535 || h > 65535) return hipErrorInvalidValue;
  if (dtype == PF_DTYPE_BF16_ && (dh == 64 || dh == 128))
    return attention_bwd_mfma(qkv, o, dout, lse, Dsum, dqkv, B, S, h, dh, causal, st);
  if (dtype == PF_DTYPE_BF16_) return launch_attn_bwd<bf16_t>(qkv, o, dout, lse, Dsum, dqkv, B, S, h, dh, causal, st);
  return launch_attn_bwd<float>(qkv, o, dout, lse, Dsum, dqkv, B, S, h, dh, causal, st);
}

hipError_t ce_loss_inplace(int32_t dtype, void* logits, const int32_t* ids, float* loss_sum, int64_t tokens,
                           int64_t pitch, int32_t V, int32_t S, float inv_n, hipStream_t st) {
  if (tokens <= 0 || pitch < V || V <= 0 || S <= 1) return hipErrorInvalidValue;
  const dim3 grid((unsigned)tokens), block(256);
  if (dtype == PF_DTYPE_BF16_ && pitch % 8 == 0 && ((uintptr_t)logits & 15) == 0) {
    hipLaunchKernelGGL(ce_loss_bf16_vec_kernel, grid, block, 0, st, (bf16_t*)logits, ids, loss_sum, pitch, V, S, inv_n);
    return hipGetLastError();
  }
  PF_BY_DTYPE(dtype,
              hipLaunchKernelGGL(ce_loss_kernel<bf16_t>, grid, block, 0, st, (bf16_t*)logits, ids, loss_sum, pitch, V, S, inv_n),
              hipLaunchKernelGGL(ce_loss_kernel<float>, grid, block, 0, st, (float*)logits, ids, loss_sum, pitch, V, S, inv_n));
  return hipGetLastError();
}

hipError_t embed_bwd(int32_t dtype, const void* dx, const int32_t* ids, float* dtok, float* dpos, int64_t tokens,
                     int32_t S, int32_t d, int32_t V, hipStream_t st) {
  if (tokens <= 0 || d % 8 != 0) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((tokens + 3) / 4)), block(256);
  PF_BY_DTYPE(dtype,
              hipLaunchKernelGGL(embed_bwd_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)dx, ids, dtok, dpos, tokens, S, d, V),
              hipLaunchKernelGGL(embed_bwd_kernel<float>, grid, block, 0, st, (const float*)dx, ids, dtok, dpos, tokens, S, d, V));
  return hipGetLastError();
}

hipError_t adam_update(float* theta, float* m, float* v, float* g, int64_t n, float lr, float b1, float b2, float eps,
                       int64_t step, int32_t accum, hipStream_t st, bool dry) {
  if (n <= 0 || step < 1 || accum < 1) return hipErrorInvalidValue;
  const float bc1 = 1.f - powf(b1, (float)step), bc2 = 1.f - powf(b2, (float)step);
  if (dry) {   // same loads, stores and arithmetic, but m, v and theta keep their values (finite gradients assumed): only g is cleared
    lr = 0.f;
    b1 = b2 = 1.f;
  }
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, theta, m, v, g, n, lr, b1, b2,
                     eps, bc1, bc2, 1.f / (float)accum);
  return hipGetLastError();
}

hipError_t cast_from_f32(int32_t dtype, const float* src, void* dst, void* dst_t, int64_t R, int64_t Cn,
                         hipStream_t st) {
  if (R <= 0 || Cn <= 0) return hipErrorInvalidValue;
  if (dst_t) {
    const dim3 grid((unsigned)((Cn + 63) / 64), (unsigned)((R + 63) / 64));
    if (grid.y > 65535) return hipErrorInvalidValue;
    PF_BY_DTYPE(dtype,
                hipLaunchKernelGGL(cast_transpose_kernel<bf16_t>, grid, dim3(256), 0, st, src, (bf16_t*)dst, (bf16_t*)dst_t, R, Cn),
                hipLaunchKernelGGL(cast_transpose_kernel<float>, grid, dim3(256), 0, st, src, (float*)dst, (float*)dst_t, R, Cn));
  } else {
    const int64_t n = R * Cn;
    const dim3 grid((unsigned)((n + 255) / 256));
    PF_BY_DTYPE(dtype, hipLaunchKernelGGL(cast_kernel<bf16_t>, grid, dim3(256), 0, st, src, (bf16_t*)dst, n),
                hipLaunchKernelGGL(cast_kernel<float>, grid, dim3(256), 0, st, src, (float*)dst, n));
  }
  return hipGetLastError();
}

hipError_t widen_to_f32(int32_t dtype, const void* src, float* dst, int64_t n, hipStream_t st) {
  if (n <= 0) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((n + 255) / 256));
  PF_BY_DTYPE(dtype, hipLaunchKernelGGL(widen_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)src, dst, n),
              hipLaunchKernelGGL(widen_kernel<float>, grid, dim3(256), 0, st, (const float*)src, dst, n));
  return hipGetLastError();
}

}  // namespace pf

// ---- LayerNorm backward without a workspace argument ---------------------------------------------------------
// The partial dg / db rows of layernorm_bwd_kernel live in a device array of the library's own instead of a buffer
// of the caller's.  The array's name is a host-side stand-in in host code: its device address is looked up once per
// device and only that pointer is handed to kernels.
namespace {
constexpr int64_t kStaticScratchBytes = (int64_t)8 << 20;
static __device__ __align__(256) float scratch[kStaticScratchBytes / 4];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;
}  // namespace

extern "C" int32_t pf_op_layernorm_bwd_static(int32_t dtype, const void* dy, const void* x, const void* g,
                                              const float* mean, const float* rstd, const void* resid, void* dx,
                                              float* dg, float* db, int64_t rows, int32_t d, void* stream) {
  if ((dtype != PF_DTYPE_F32 && dtype != PF_DTYPE_BF16) || !dy || !x || !g || !mean || !rstd || !dx || !dg || !db ||
      rows <= 0 || d <= 0 || d % 8 != 0)
    return pf::fail(PF_ERR_ARG, "pf_op_layernorm_bwd_static: bad argument");
  if (d > 8192)
    return pf::fail(PF_ERR_ARG, "pf_op_layernorm_bwd_static: d = %d exceeds the maximum of 8192 columns", d);
  // one partial row is 2 * d floats; the array holds at least 128 of them at the widest d
  int64_t max_blocks = kStaticScratchBytes / (2 * (int64_t)d * 4);
  if (max_blocks > pf::LN_BWD_MAX_BLOCKS * 4) max_blocks = pf::LN_BWD_MAX_BLOCKS * 4;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return pf::fail(PF_ERR_HIP, "pf_op_layernorm_bwd_static: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return pf::fail(PF_ERR_ARG, "pf_op_layernorm_bwd_static: device index %d not supported", dev);
  float* ptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {   // first call on this device, which is the current one: its copy of the array
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return pf::fail(PF_ERR_HIP, "pf_op_layernorm_bwd_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
      g_scratch_ptr[dev] = (float*)p;
    }
    ptr = g_scratch_ptr[dev];
  }
  // every partial row the second kernel reads is written by the first in the same call: nothing to clear
  e = pf::layernorm_bwd(dtype, dy, x, g, mean, rstd, resid, dx, dg, db, ptr, rows, d, (hipStream_t)stream, max_blocks);
  if (e != hipSuccess) return pf::fail(PF_ERR_HIP, "pf_op_layernorm_bwd_static: %s", hipGetErrorString(e));
  return PF_OK;
}
