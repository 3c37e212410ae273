// Attention backward for bf16, d_head 64 or 128, on the 32x32x16 bf16 MFMA (gfx950).
//
// With P = exp(scale * Q K^T - lse), dP = dO V^T, dS = P * (dP - D), D[q] = sum_j dO[q][j] O[q][j]:
//   dV = P^T dO,   dK = scale * dS^T Q,   dQ = scale * dS K.
// Two passes, each owning its outputs (no atomics, deterministic):
//  * dK/dV pass: a workgroup owns 128 keys (32 per wave, their K and V rows live in registers as
//    MFMA "B" operands) and walks the queries in tiles of 64 staged in LDS.  S = Q K^T and dP = dO V^T
//    are computed with the query tile as the "A" operand, so a lane holds ONE key and 32 of the 64
//    queries: exactly the "B" operand layout the second pair of products needs
//    (dV^T += dO^T P, dK^T += Q^T dS, contraction over queries), with Q^T and dO^T fragments read from
//    the same row-major tiles through the transposing LDS load (ds_read_b64_tr_b16).
//  * dQ pass: mirror image of the forward kernel: a workgroup owns 128 queries (Q and dO rows in
//    registers), walks the keys in tiles of 64; S^T = K Q^T and dP^T = V dO^T put one query per lane,
//    so lse and D are per-lane scalars, and dQ^T += K^T dS^T reads K^T through the transposing load.
// Tiles go global -> LDS directly (no staging registers), a whole tile ahead, into the other of two buffers.
// A small pre-pass computes D.
#include "pf_kernels.h"
#include "pf_device.h"


namespace pf {
namespace {

constexpr float LOG2E_B = 1.4426950408889634f;

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

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(3))) char* lds_char_ptr;

// Tiles of 64 rows x d_head lie in LDS row-major, as in memory, with the 16-byte chunks of a row XOR-swizzled by
// swz_rt(row).  A tile is read two ways: row-wise (one 16-byte chunk per lane, consecutive rows per lane: the MFMA
// operand whose contraction runs over d_head) and through the transposing LDS load (16 lanes fetch a 4-row x
// 32-byte block: the operand whose contraction runs over the rows).  The swizzle is a bijection of the 16 (d_head
// 128) or 8 (d_head 64, two rows per 256 bytes) bank phases for the first, and moves the 32-byte pairs of four
// consecutive rows apart for the second.  It depends on row % 16 only.
template <int CPR>
__device__ __forceinline__ int swz_rt(int r) {
  if (CPR == 8) {
    const int x = (r >> 1) & 7;
    return ((x & 1) << 1) | ((x >> 1) & 1) | (x & 4);
  }
  const int x = r & 15;
  return (x & 8) | ((x & 3) << 1) | ((x >> 2) & 1);
}

// one wave-wide copy of 1 KB, global -> LDS directly: lane i's 16 bytes land at dst + 16 i (dst wave-uniform)
__device__ __forceinline__ void copy_1k(uint32_t dst, const bf16_t* p) {
  lds_direct_load_1k(dst, p);
}

// Byte offsets of a lane's transposing reads inside a tile, for the 32-column block dt and K step 0: lane 16 G + p
// points at row 8 r + 4 g + p / 4 (r = 0, 1: the two reads; g = lane / 32) and at the four columns from
// 32 dt + 16 (G % 2) + 4 (p % 4), and receives column 32 dt + lane % 32 of the four rows.  K step i adds 16 i rows
// (the swizzle has period 16); the two reads are 8 rows apart, where the swizzle differs, so both offsets are kept.
template <int DH>
__device__ __forceinline__ void tr_offsets(int lane, int off[][2]) {
  constexpr int CPR = DH / 8, ROWB = DH * 2;
  const int pl = lane & 15, mb = (lane >> 4) & 1, g = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int row = 8 * r + 4 * g + (pl >> 2);
      const int c = dt * 4 + mb * 2 + ((pl & 3) >> 1);
      off[dt][r] = row * ROWB + ((c ^ swz_rt<CPR>(row)) << 4) + 8 * (pl & 1);
    }
}

template <int ROWB>
__device__ __forceinline__ bf16x8 read_tr_frag2(lds_char_ptr tile, const int off[2], int i) {
  const v4s r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(tile + off[0] + 16 * i * ROWB));
  const v4s r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(tile + off[1] + 16 * i * ROWB));
  v8s f;
  f[0] = r0[0]; f[1] = r0[1]; f[2] = r0[2]; f[3] = r0[3];
  f[4] = r1[0]; f[5] = r1[1]; f[6] = r1[2]; f[7] = r1[3];
  return __builtin_bit_cast(bf16x8, f);
}

// ------------------------------------------------------------------------------------------------
// dK, dV: a workgroup owns 128 keys (a wave 32 of them, K and V fragments in registers) and walks the queries in
// tiles of 64.  Per tile: Q and dO go global -> LDS directly, a whole tile ahead, into the other of two buffers;
// lse and D of the tile travel through one register per thread.
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 2 : 1) void attn_bwd_dkv_bf16_kernel(const bf16_t* __restrict__ qkv,
                                                                const bf16_t* __restrict__ dout,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv,
                                                                int32_t S, int32_t h, int32_t causal, float scale_log2e,
                                                                float scale, int32_t nblk, int32_t n_wg,
                                                                int32_t alternate) {
  constexpr int CPR = DH / 8, KS = DH / 16, DT = DH / 32, ROWB = DH * 2, TILE = 64 * ROWB, NI = TILE / 1024,
                RPI = 1024 / ROWB;
  constexpr int BUF = 2 * TILE + 512;   // Q tile | dO tile | lse (log2 units) of the 64 queries | D
  extern __shared__ __align__(16) char dyn_smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5;
  // the key blocks of one (batch, head) run on one XCD: they all re-read that head's Q and dO
  const int unit = (int)xcd_contiguous(blockIdx.x, n_wg);
  const int b = unit / (nblk * h), hd = (unit / nblk) % h;
  // Causal: the early key blocks are the long ones.  Workgroups whose ids are 256 apart share a CU; `alternate`
  // (every 32 consecutive units of an XCD's range are whole heads, the launcher checks) hands every other such group
  // out in the opposite order, so that a CU holds a long and a short block rather than two of one length.
  int kpos = unit % nblk;
  if (alternate && ((blockIdx.x >> 8) & 1)) kpos = nblk - 1 - kpos;
  const int k_blk = kpos * 128;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;
  const uint32_t rs32 = (uint32_t)rs, d32 = (uint32_t)d;
  const bf16_t* base = qkv + (int64_t)b * S * rs + hd * DH;
  const bf16_t* dobase = dout + (int64_t)b * S * d + hd * DH;
  const int key = k_blk + wave * 32 + lr;

  // rows past the end are clamped, not branched around (a load in a branch makes the compiler wait for everything
  // in flight at the join); what a clamped key accumulates is not stored
  bf16x8 fk[KS], fv[KS];
  {
    const bf16_t* p = base + (uint64_t)(uint32_t)(key < S ? key : S - 1) * rs32 + g * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      fk[kk] = as_bf16x8(*(const uint4*)(p + d + kk * 16));
      fv[kk] = as_bf16x8(*(const uint4*)(p + 2 * d + kk * 16));
    }
  }
  f32x16 accK[DT], accV[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) accK[i][r] = accV[i][r] = 0.f;

  const int st_row = wave * RPI + lane / CPR;
  const int st_col = ((lane % CPR) ^ swz_rt<CPR>(st_row)) << 3;   // the same for all copies of a lane (rows 16 apart)
  static_assert((4 * RPI) % 16 == 0, "rows of one lane's copies must share their swizzle");
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_ptr)dyn_smem);
  auto stage = [&](int buf, int q0) {
#pragma unroll
    for (int i = 0; i < NI / 4; ++i) {
      int row = q0 + st_row + 4 * i * RPI;
      row = row < S ? row : S - 1;
      const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)(buf * BUF + (wave + 4 * i) * 1024));
      copy_1k(dst, base + (uint64_t)(uint32_t)row * rs32 + st_col);
      copy_1k(dst + TILE, dobase + (uint64_t)(uint32_t)row * d32 + st_col);
    }
  };
  // threads 0..63 carry lse, 64..127 carry D (the others repeat them and write nothing)
  const float* ld_src = ((tid & 64) ? Dsum : lse) + ((int64_t)b * h + hd) * S;
  auto load_ld = [&](int q0) {
    const int q = q0 + (tid & 63);
    return ld_src[q < S ? q : S - 1];
  };
  auto write_ld = [&](int buf, int q0, float v) {
    if (tid < 128) {
      const bool ok = q0 + (tid & 63) < S;
      // a query past the end gets lse = +inf, so its probabilities are exp2(x - inf) = 0
      const float w = (tid < 64) ? (ok ? v * LOG2E_B : INFINITY) : (ok ? v : 0.f);
      *(float*)(dyn_smem + buf * BUF + 2 * TILE + tid * 4) = w;
    }
  };
  int t_off[DT][2];
  tr_offsets<DH>(lane, t_off);

  const int n_qt = (S + 63) / 64;
  const int qt0 = causal ? k_blk / 64 : 0;   // queries before the first key of the block see none of its keys
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) asm volatile("" ::"v"(fk[kk]), "v"(fv[kk]));   // waited for here, once
  float ld = 0.f;
  if (qt0 < n_qt) {
    stage(0, qt0 * 64);
    ld = load_ld(qt0 * 64);
  }
  for (int qt = qt0; qt < n_qt; ++qt) {
    const int cur = (qt - qt0) & 1, q0 = qt * 64;
    // buffer cur was last read two iterations ago and the barrier of the previous iteration is behind us
    write_ld(cur, q0, ld);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (qt + 1 < n_qt) {
      stage(cur ^ 1, q0 + 64);
      ld = load_ld(q0 + 64);
    }
    const char* sQ = dyn_smem + cur * BUF;
    const char* sdO = sQ + TILE;
    const float* sL = (const float*)(sQ + 2 * TILE);
    const float* sD = sL + 64;
    lds_char_ptr tQ = (lds_char_ptr)(lds_void_ptr)dyn_smem + cur * BUF;
    lds_char_ptr tdO = tQ + TILE;

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
        const int o = r * ROWB + ((c ^ swz_rt<CPR>(r)) << 4);
        aS = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(const uint4*)(sQ + o)), fk[kk], aS, 0, 0, 0);
        aP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(const uint4*)(sdO + o)), fv[kk], aP, 0, 0, 0);
      }
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int qi = qs * 32 + 8 * rg + 4 * g;
        const float4 L4 = *(const float4*)(sL + qi);
        const float4 D4 = *(const float4*)(sD + qi);
        const float Lv[4] = {L4.x, L4.y, L4.z, L4.w}, Dv[4] = {D4.x, D4.y, D4.z, D4.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float p = __builtin_amdgcn_exp2f(fmaf(aS[rg * 4 + j], scale_log2e, -Lv[j]));
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
        accV[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr_frag2<ROWB>(tdO, t_off[dt], i), fp, accV[dt], 0, 0, 0);
        accK[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr_frag2<ROWB>(tQ, t_off[dt], i), fds, accK[dt], 0, 0, 0);
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
// dQ: a workgroup owns 128 queries (Q and dO fragments, lse and D in registers) and walks the keys in tiles of
// 64; K and V tiles go global -> LDS directly, a whole tile ahead, into the other of two buffers.
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void attn_bwd_dq_bf16_kernel(const bf16_t* __restrict__ qkv,
                                                               const bf16_t* __restrict__ dout,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv,
                                                               int32_t S, int32_t h, int32_t causal, float scale_log2e,
                                                               float scale, int32_t nblk, int32_t n_wg,
                                                               int32_t alternate) {
  constexpr int CPR = DH / 8, KS = DH / 16, DT = DH / 32, ROWB = DH * 2, TILE = 64 * ROWB, NI = TILE / 1024,
                RPI = 1024 / ROWB;
  constexpr int BUF = 2 * TILE;   // K tile | V tile
  extern __shared__ __align__(16) char dyn_smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5;
  // the query blocks of one (batch, head) run on one XCD: they all re-read that head's K and V
  const int unit = (int)xcd_contiguous(blockIdx.x, n_wg);
  const int b = unit / (nblk * h), hd = (unit / nblk) % h;
  // causal: the long (late) blocks start first; `alternate` as in the dK/dV pass
  int qpos = unit % nblk;
  if (alternate && ((blockIdx.x >> 8) & 1)) qpos = nblk - 1 - qpos;
  const int q_blk = (causal ? nblk - 1 - qpos : qpos) * 128;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;
  const uint32_t rs32 = (uint32_t)rs;
  const bf16_t* base = qkv + (int64_t)b * S * rs + hd * DH;
  const int q_row = q_blk + wave * 32 + lr;
  const bool live = q_row < S;
  const int q_cl = live ? q_row : S - 1;

  bf16x8 fq[KS], fdo[KS];
  {
    const bf16_t* pq = base + (uint64_t)(uint32_t)q_cl * rs32 + g * 8;
    const bf16_t* pd = dout + ((int64_t)b * S + q_cl) * d + hd * DH + g * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      fq[kk] = as_bf16x8(*(const uint4*)(pq + kk * 16));
      fdo[kk] = as_bf16x8(*(const uint4*)(pd + kk * 16));
    }
  }
  const float Lraw = lse[((int64_t)b * h + hd) * S + q_cl], Draw = Dsum[((int64_t)b * h + hd) * S + q_cl];
  const float nLq = live ? -Lraw * LOG2E_B : -INFINITY;   // a query past the end: exp2(x - inf) = 0
  const float Dq = live ? Draw : 0.f;
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
  const int st_row = wave * RPI + lane / CPR;
  const int st_col = ((lane % CPR) ^ swz_rt<CPR>(st_row)) << 3;
  static_assert((4 * RPI) % 16 == 0, "rows of one lane's copies must share their swizzle");
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_ptr)dyn_smem);
  auto stage = [&](int buf, int k0) {
#pragma unroll
    for (int i = 0; i < NI / 4; ++i) {
      int row = k0 + st_row + 4 * i * RPI;
      row = row < S ? row : S - 1;
      const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)(buf * BUF + (wave + 4 * i) * 1024));
      const bf16_t* p = base + (uint64_t)(uint32_t)row * rs32 + st_col;
      copy_1k(dst, p + d);
      copy_1k(dst + TILE, p + 2 * d);
    }
  };
  int t_off[DT][2];
  tr_offsets<DH>(lane, t_off);
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) asm volatile("" ::"v"(fq[kk]), "v"(fdo[kk]));   // waited for here, once
  asm volatile("" ::"v"(nLq), "v"(Dq));

  stage(0, 0);
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int k0 = kt * 64, cur = kt & 1;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + 1 < n_tiles) stage(cur ^ 1, k0 + 64);
    const char* sK = dyn_smem + cur * BUF;
    const char* sV = sK + TILE;
    lds_char_ptr tK = (lds_char_ptr)(lds_void_ptr)dyn_smem + cur * BUF;
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
        const int o = r * ROWB + ((c ^ swz_rt<CPR>(r)) << 4);
        aS = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(const uint4*)(sK + o)), fq[kk], aS, 0, 0, 0);
        aP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*(const uint4*)(sV + o)), fdo[kk], aP, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(fmaf(aS[r], scale_log2e, nLq));
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
      for (int dt = 0; dt < DT; ++dt)
        accQ[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr_frag2<ROWB>(tK, t_off[dt], i), fds, accQ[dt], 0, 0, 0);
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
  constexpr int TILE = 64 * DH * 2;
  constexpr size_t lds_dkv = 2 * (2 * TILE + 512), lds_dq = 2 * 2 * TILE;   // two buffers each
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_bwd_dkv_bf16_kernel<DH>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_dkv);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)attn_bwd_dq_bf16_kernel<DH>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_dq);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // groups of 32 consecutive units of an XCD's range must be whole heads for the reversal to permute units
  // (MI355X: 569 -> 527 us on 256 heads of 1024 tokens with d_head 128, 152 -> 148 us on 128 heads with d_head 64)
  const int32_t alternate = (causal && nblk > 1 && 32 % nblk == 0 && n_wg % 8 == 0 && (n_wg / 8) % 32 == 0) ? 1 : 0;
  hipLaunchKernelGGL(attn_bwd_dkv_bf16_kernel<DH>, grid, block, lds_dkv, st, (const bf16_t*)qkv, (const bf16_t*)dout,
                     lse, Dsum, (bf16_t*)dqkv, S, h, causal, scale * LOG2E_B, scale, (int32_t)nblk, (int32_t)n_wg, alternate);
  hipLaunchKernelGGL(attn_bwd_dq_bf16_kernel<DH>, grid, block, lds_dq, st, (const bf16_t*)qkv, (const bf16_t*)dout, lse,
                     Dsum, (bf16_t*)dqkv, S, h, causal, scale * LOG2E_B, scale, (int32_t)nblk, (int32_t)n_wg, alternate);
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
