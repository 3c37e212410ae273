// Attention backward for bf16, d_head 64 or 128, on the 32x32x16 bf16 MFMA (gfx950).
//
// With P = exp(scale * Q K^T - lse), dP = dO V^T, dS = P * (dP - D), D[q] = sum_j dO[q][j] O[q][j]:
//   dV = P^T dO,   dK = scale * dS^T Q,   dQ = scale * dS K.
// Two passes, each owning its outputs (no atomics, deterministic):
//  * dK/dV pass: a workgroup owns 128 keys (32 per wave, their K and V rows live in registers as
//    MFMA "B" operands) and walks the queries in tiles of 64 staged in LDS.  S = Q K^T and dP = dO V^T
//    are computed with the query tile as the "A" operand, so a lane holds ONE key and 32 of the 64
//    queries: exactly the "B" operand layout the second pair of products needs
//    (dV^T += dO^T P, dK^T += Q^T dS, contraction over queries), with Q^T and dO^T read from
//    transposed copies of the tile in LDS.
//  * dQ pass: mirror image of the forward kernel: a workgroup owns 128 queries (Q and dO rows in
//    registers), walks the keys in tiles of 64; S^T = K Q^T and dP^T = V dO^T put one query per lane,
//    so lse and D are per-lane scalars, and dQ^T += K^T dS^T reads K^T from a transposed LDS copy.
// A small pre-pass computes D.
#include "pf_kernels.h"
#include "pf_device.h"

namespace pf {
namespace {

constexpr float LOG2E_B = 1.4426950408889634f;

template <int CPR>
__device__ __forceinline__ int swz(int r, int c) {
  return (CPR == 8) ? (c ^ ((r >> 1) & 7)) : (c ^ (r & 15));
}

// D[b][h][q] = sum_j dO[q][j] * O[q][j]
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_prep_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                                            float* __restrict__ Dsum, int32_t B, int32_t S, int32_t h) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over B * S * h
  if (idx >= (int64_t)B * S * h) return;
  const int hd = (int)(idx % h);
  const int64_t t = idx / h;
  const int d = h * DH;
  const bf16_t* po = o + t * d + hd * DH;
  const bf16_t* pd = dout + t * d + hd * DH;
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < DH; c += 8) {
    float a[8], b[8];
    load8(po + c, a);
    load8(pd + c, b);
#pragma unroll
    for (int j = 0; j < 8; ++j) s = fmaf(a[j], b[j], s);
  }
  const int64_t bb = t / S, q = t % S;
  Dsum[(bb * h + hd) * S + q] = s;
}

// stage a 64-row tile of one head: `rows` valid rows starting at src (row stride rs elements) into a
// swizzled [row][dh] copy and, if dstT is given, a transposed [dh][row] copy with pitch 68
template <int DH>
__device__ __forceinline__ void stage_tile(const bf16_t* src, int64_t rs, int rows, uint4* dst, uint16_t* dstT, int tid) {
  constexpr int CPR = DH / 8;
#pragma unroll
  for (int i = 0; i < 64 * CPR / 256; ++i) {
    const int q = tid + i * 256, r = q / CPR, c = q % CPR;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < rows) v = *(const uint4*)(src + (int64_t)r * rs + c * 8);
    dst[r * CPR + swz<CPR>(r, c)] = v;
    if (dstT) {
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        dstT[(c * 8 + 2 * j) * 68 + r] = (uint16_t)(w[j] & 0xffffu);
        dstT[(c * 8 + 2 * j + 1) * 68 + r] = (uint16_t)(w[j] >> 16);
      }
    }
  }
}

__device__ __forceinline__ bf16x8 read_t_frag(const uint16_t* rowp) {
  const uint2 lo = *(const uint2*)rowp;
  const uint2 hi = *(const uint2*)(rowp + 8);
  return as_bf16x8(make_uint4(lo.x, lo.y, hi.x, hi.y));
}

// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 2 : 1) void attn_bwd_dkv_bf16_kernel(const bf16_t* __restrict__ qkv,
                                                                const bf16_t* __restrict__ dout,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv,
                                                                int32_t S, int32_t h, int32_t causal, float scale_log2e,
                                                                float scale, int32_t nblk, int32_t n_wg) {
  constexpr int CPR = DH / 8, KS = DH / 16, DT = DH / 32, TP = 68;
  // dynamic LDS (68 KB for d_head 128): Q | dO tiles, their transposes, lse and D of the tile
  extern __shared__ uint4 dyn_smem[];
  uint4* sQ = dyn_smem;
  uint4* sdO = sQ + 64 * CPR;
  uint16_t* sQt = (uint16_t*)(sdO + 64 * CPR);
  uint16_t* sdOt = sQt + DH * TP;
  float* sL = (float*)(sdOt + DH * TP);
  float* sD = sL + 64;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5;
  // the key blocks of one (batch, head) run on one XCD: they all re-read that head's Q and dO
  const int unit = (int)xcd_contiguous(blockIdx.x, n_wg);
  const int b = unit / (nblk * h), hd = (unit / nblk) % h;
  const int k_blk = (unit % nblk) * 128;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;
  const bf16_t* base = qkv + (int64_t)b * S * rs + hd * DH;
  const bf16_t* dobase = dout + (int64_t)b * S * d + hd * DH;
  const int key = k_blk + wave * 32 + lr;

  bf16x8 fk[KS], fv[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    uint4 a = make_uint4(0, 0, 0, 0), c = make_uint4(0, 0, 0, 0);
    if (key < S) {
      const bf16_t* p = base + (int64_t)key * rs + kk * 16 + g * 8;
      a = *(const uint4*)(p + d);
      c = *(const uint4*)(p + 2 * d);
    }
    fk[kk] = as_bf16x8(a);
    fv[kk] = as_bf16x8(c);
  }
  f32x16 accK[DT], accV[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) accK[i][r] = accV[i][r] = 0.f;

  const int n_qt = (S + 63) / 64;
  const int qt0 = causal ? k_blk / 64 : 0;   // queries before the first key of the block see none of its keys
  for (int qt = qt0; qt < n_qt; ++qt) {
    const int q0 = qt * 64;
    const int rows = (S - q0 < 64) ? S - q0 : 64;
    __syncthreads();
    stage_tile<DH>(base + (int64_t)q0 * rs, rs, rows, sQ, sQt, tid);
    stage_tile<DH>(dobase + (int64_t)q0 * d, d, rows, sdO, sdOt, tid);
    if (tid < 64) {
      const bool ok = tid < rows;
      sL[tid] = ok ? lse[((int64_t)b * h + hd) * S + q0 + tid] * LOG2E_B : INFINITY;   // exp2(x - inf) = 0
      sD[tid] = ok ? Dsum[((int64_t)b * h + hd) * S + q0 + tid] : 0.f;
    }
    __syncthreads();

    f32x16 P[2], dS[2];
    const bool need_mask = causal && (q0 < k_blk + 128);
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      f32x16 aS, aP;
#pragma unroll
      for (int r = 0; r < 16; ++r) aS[r] = aP[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        const int r = qs * 32 + lr, c = kk * 2 + g;
        const int o = r * CPR + swz<CPR>(r, c);
        aS = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(sQ[o]), fk[kk], aS, 0, 0, 0);
        aP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(sdO[o]), fv[kk], aP, 0, 0, 0);
      }
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int qi = qs * 32 + 8 * rg + 4 * g;
        const float4 L4 = *(const float4*)(sL + qi);
        const float4 D4 = *(const float4*)(sD + qi);
        const float Lv[4] = {L4.x, L4.y, L4.z, L4.w}, Dv[4] = {D4.x, D4.y, D4.z, D4.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float p = __builtin_amdgcn_exp2f(aS[rg * 4 + j] * scale_log2e - Lv[j]);
          if (need_mask && key > q0 + qi + j) p = 0.f;
          P[qs][rg * 4 + j] = p;
          dS[qs][rg * 4 + j] = p * (aP[rg * 4 + j] - Dv[j]);
        }
      }
    }
    // contraction over the 64 queries: K step i covers queries 16i..16i+15, operand slot (g, t) is
    // query 16i + 8*(t/4) + 4g + t%4 = register 8*(i%2) + t of sub-tile i/2
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x8 fp, fds;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        fp[t] = (__bf16)P[i >> 1][8 * (i & 1) + t];
        fds[t] = (__bf16)dS[i >> 1][8 * (i & 1) + t];
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const int off = (dt * 32 + lr) * TP + 16 * i + 4 * g;
        accV[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t_frag(sdOt + off), fp, accV[dt], 0, 0, 0);
        accK[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t_frag(sQt + off), fds, accK[dt], 0, 0, 0);
      }
    }
  }
  if (key < S) {
    bf16_t* orow = dqkv + ((int64_t)b * S + key) * rs + hd * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const float vk[4] = {accK[dt][rg * 4] * scale, accK[dt][rg * 4 + 1] * scale, accK[dt][rg * 4 + 2] * scale,
                             accK[dt][rg * 4 + 3] * scale};
        const float vv[4] = {accV[dt][rg * 4], accV[dt][rg * 4 + 1], accV[dt][rg * 4 + 2], accV[dt][rg * 4 + 3]};
        store4(orow + d + dt * 32 + rg * 8 + g * 4, vk);
        store4(orow + 2 * d + dt * 32 + rg * 8 + g * 4, vv);
      }
  }
}

// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void attn_bwd_dq_bf16_kernel(const bf16_t* __restrict__ qkv,
                                                               const bf16_t* __restrict__ dout,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv,
                                                               int32_t S, int32_t h, int32_t causal, float scale_log2e,
                                                               float scale, int32_t nblk, int32_t n_wg) {
  constexpr int CPR = DH / 8, KS = DH / 16, DT = DH / 32, TP = 68;
  __shared__ uint4 sK[64 * CPR];
  __shared__ uint4 sV[64 * CPR];
  __shared__ uint16_t sKt[DH * TP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5;
  // the query blocks of one (batch, head) run on one XCD: they all re-read that head's K and V
  const int unit = (int)xcd_contiguous(blockIdx.x, n_wg);
  const int b = unit / (nblk * h), hd = (unit / nblk) % h;
  const int q_blk = (unit % nblk) * 128;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;
  const bf16_t* base = qkv + (int64_t)b * S * rs + hd * DH;
  const int q_row = q_blk + wave * 32 + lr;
  const bool live = q_row < S;

  bf16x8 fq[KS], fdo[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    uint4 a = make_uint4(0, 0, 0, 0), c = make_uint4(0, 0, 0, 0);
    if (live) {
      a = *(const uint4*)(base + (int64_t)q_row * rs + kk * 16 + g * 8);
      c = *(const uint4*)(dout + ((int64_t)b * S + q_row) * d + hd * DH + kk * 16 + g * 8);
    }
    fq[kk] = as_bf16x8(a);
    fdo[kk] = as_bf16x8(c);
  }
  const float Lq = live ? lse[((int64_t)b * h + hd) * S + q_row] * LOG2E_B : INFINITY;
  const float Dq = live ? Dsum[((int64_t)b * h + hd) * S + q_row] : 0.f;
  f32x16 accQ[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) accQ[i][r] = 0.f;

  int n_tiles = (S + 63) / 64;
  if (causal) {
    const int last_q = (q_blk + 127 < S - 1) ? q_blk + 127 : S - 1;
    const int need = last_q / 64 + 1;
    if (need < n_tiles) n_tiles = need;
  }
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int k0 = kt * 64;
    const int rows = (S - k0 < 64) ? S - k0 : 64;
    __syncthreads();
    stage_tile<DH>(base + (int64_t)k0 * rs + d, rs, rows, sK, sKt, tid);
    stage_tile<DH>(base + (int64_t)k0 * rs + 2 * d, rs, rows, sV, nullptr, tid);
    __syncthreads();
    const bool need_mask = (k0 + 63 >= S) || (causal && k0 + 63 > q_blk + wave * 32);
    f32x16 dS[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      f32x16 aS, aP;
#pragma unroll
      for (int r = 0; r < 16; ++r) aS[r] = aP[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        const int r = ks * 32 + lr, c = kk * 2 + g;
        const int o = r * CPR + swz<CPR>(r, c);
        aS = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(sK[o]), fq[kk], aS, 0, 0, 0);
        aP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(sV[o]), fdo[kk], aP, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(aS[r] * scale_log2e - Lq);
        if (need_mask) {
          const int key = k0 + ks * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (key >= S || (causal && key > q_row)) p = 0.f;
        }
        dS[ks][r] = p * (aP[r] - Dq);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x8 fds;
#pragma unroll
      for (int t = 0; t < 8; ++t) fds[t] = (__bf16)dS[i >> 1][8 * (i & 1) + t];
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const int off = (dt * 32 + lr) * TP + 16 * i + 4 * g;
        accQ[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t_frag(sKt + off), fds, accQ[dt], 0, 0, 0);
      }
    }
  }
  if (live) {
    bf16_t* orow = dqkv + ((int64_t)b * S + q_row) * rs + hd * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const float v[4] = {accQ[dt][rg * 4] * scale, accQ[dt][rg * 4 + 1] * scale, accQ[dt][rg * 4 + 2] * scale,
                            accQ[dt][rg * 4 + 3] * scale};
        store4(orow + dt * 32 + rg * 8 + g * 4, v);
      }
  }
}

template <int DH>
hipError_t launch(const void* qkv, const void* o, const void* dout, const float* lse, float* Dsum, void* dqkv,
                  int32_t B, int32_t S, int32_t h, int32_t causal, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)DH);
  const int64_t n = (int64_t)B * S * h;
  hipLaunchKernelGGL(attn_bwd_prep_kernel<DH>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const bf16_t*)o,
                     (const bf16_t*)dout, Dsum, B, S, h);
  const int64_t nblk = (S + 127) / 128, n_wg = nblk * h * B;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)n_wg), block(256);
  constexpr size_t lds = 2 * 64 * (DH / 8) * 16 + 2 * DH * 68 * 2 + 2 * 64 * 4;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_bwd_dkv_bf16_kernel<DH>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(attn_bwd_dkv_bf16_kernel<DH>, grid, block, lds, st, (const bf16_t*)qkv, (const bf16_t*)dout, lse,
                     Dsum, (bf16_t*)dqkv, S, h, causal, scale * LOG2E_B, scale, (int32_t)nblk, (int32_t)n_wg);
  hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel<DH>, grid, block, 0, st, (const bf16_t*)qkv, (const bf16_t*)dout, lse, Dsum,
                     (bf16_t*)dqkv, S, h, causal, scale * LOG2E_B, scale, (int32_t)nblk, (int32_t)n_wg);
  return hipGetLastError();
}

}  // namespace

hipError_t attention_bwd_mfma(const void* qkv, const void* o, const void* dout, const float* lse, float* Dsum, void* dqkv,
                              int32_t B, int32_t S, int32_t h, int32_t dh, int32_t causal, hipStream_t st) {
  if (dh == 64) return launch<64>(qkv, o, dout, lse, Dsum, dqkv, B, S, h, causal, st);
  if (dh == 128) return launch<128>(qkv, o, dout, lse, Dsum, dqkv, B, S, h, causal, st);
  return hipErrorInvalidValue;
}

}  // namespace pf
