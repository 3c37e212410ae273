// Attention forward for gfx950.
//
// bf16, d_head 64 or 128: flash-style kernel.  A workgroup of 4 waves owns 128 queries of one
// (batch, head); each wave owns 32 of them and walks the keys in tiles of 64 staged in LDS.  The
// kernel computes S^T = K Q^T with the 32x32x16 bf16 MFMA (K tile rows are the "A" operand, the
// wave's Q rows the "B" operand, kept in registers), so that a lane holds 32 of the 64 scores of ONE
// query: running max / sum need a single cross-lane exchange (lane ^ 32) and the rescale factor
// is a per-lane scalar.  The probabilities, already in the "B" operand layout, then feed
// O^T = V^T P^T; V is transposed into LDS ([d_head][key], padded pitch) when the tile is staged so
// that the "A" operand reads are two 8-byte LDS loads.
//
// Generic path (fp32, or any d_head in {8,16,32,64,128}): one thread per query, keys staged in LDS,
// online softmax key by key.  Used for the small fp32 parity workload and odd head sizes.
#include "pf_kernels.h"
#include "pf_device.h"

namespace pf {
namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
// first-class 16-byte value (the struct type would travel through a private-memory copy)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, DH == 64 ? 3 : 2) void attn_fwd_bf16_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                            float* __restrict__ lse, int32_t S, int32_t h,
                                                            int32_t causal, float scale_log2e, int32_t nq,
                                                            int32_t n_wg) {
  constexpr int CPR = DH / 8;        // 16-byte chunks per K row
  constexpr int KS = DH / 16;        // MFMA K steps over d_head
  constexpr int DT = DH / 32;        // 32-row tiles of O^T
  constexpr int VP = 68;             // pitch (elements) of a V^T row: 64 keys + 4 pad
  constexpr int KCH = 64 * CPR / 256;   // K chunks staged per thread
  constexpr int VUNITS = 16 * CPR;      // (4-key group, chunk) units of the V transpose, one per thread
  __shared__ uint4 sK2[2][64 * CPR];                        // two tiles: one is read while the next is written
  __shared__ __align__(16) uint16_t sVt2[2][DH * VP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5;
  // Workgroup ids are dealt round-robin to the 8 XCDs; remapped so that each XCD gets a contiguous range of
  // (batch, head, query block) units, the query blocks of one head run on one XCD and its L2 serves their
  // repeated reads of that head's K and V.
  const int unit = (int)xcd_contiguous(blockIdx.x, n_wg);
  const int b = unit / (nq * h), hd = (unit / nq) % h;
  const int q_blk = (unit % nq) * 128;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;                       // row stride of qkv
  const bf16_t* base = qkv + (int64_t)b * S * rs + hd * DH;
  const int q_row = q_blk + wave * 32 + lr;                // this lane's query

  // Rows are addressed by a 32-bit row number times the row stride, clamped to the last row of the sequence, so
  // that no load sits in a branch (the compiler would otherwise wait for all of them at the next join): what a
  // clamped row brings in is masked (scores) or zeroed before it reaches LDS (V).
  const uint32_t rs32 = (uint32_t)rs;
  bf16x8 fq[KS];
  {
    const bf16_t* qp = base + (uint64_t)(uint32_t)(q_row < S ? q_row : S - 1) * rs32 + g * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) fq[kk] = as_bf16x8(*(const uint4*)(qp + kk * 16));
  }

  f32x16 accO[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) accO[i][r] = 0.f;
  int n_tiles = (S + 63) / 64;
  if (causal) {
    const int last_q = (q_blk + 127 < S - 1) ? q_blk + 127 : S - 1;
    const int need = last_q / 64 + 1;
    if (need < n_tiles) n_tiles = need;
  }

  // Tile staging goes global -> registers (issued a whole tile ahead, so the loads are in flight during
  // the previous tile's work) -> LDS (two buffers, one barrier per tile).  K keeps its row-major chunks (swizzled).  V is transposed
  // on the way: a thread takes one 8-wide d_head chunk of FOUR consecutive keys and writes, for each
  // of the 8 d_head rows, the 4 keys as one 8-byte piece; 16 lanes with consecutive key groups cover
  // 128 contiguous bytes of a V^T row, so the LDS writes are free of bank conflicts.
  const int v_kg = tid & 15, v_c = tid >> 4;
  u32x4 rk[KCH], rv[4];
  auto load_regs = [&](int k0) {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int q = tid + i * 256, r = q / CPR, c = q % CPR;
      const int row = (k0 + r < S) ? k0 + r : S - 1;
      rk[i] = *(const u32x4*)(base + (uint64_t)(uint32_t)row * rs32 + d + c * 8);
    }
    if (tid < VUNITS) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int key = k0 + 4 * v_kg + j;
        rv[j] = *(const u32x4*)(base + (uint64_t)(uint32_t)(key < S ? key : S - 1) * rs32 + 2 * d + v_c * 8);
      }
    }
  };
  auto write_lds = [&](int buf, int k0) {
    uint4* sK = sK2[buf];
    uint16_t* sVt = sVt2[buf];
    if (k0 + 64 > S && tid < VUNITS) {   // ragged last tile: keys past the end contribute 0 * 0, not 0 * V[S-1]
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (k0 + 4 * v_kg + j >= S) rv[j] = u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int q = tid + i * 256, r = q / CPR, c = q % CPR;
      const int sw = (CPR == 8) ? (c ^ ((r >> 1) & 7)) : (c ^ (r & 15));
      *(u32x4*)&sK[r * CPR + sw] = rk[i];
    }
    if (tid < VUNITS) {
      const uint32_t w0[4] = {rv[0].x, rv[0].y, rv[0].z, rv[0].w}, w1[4] = {rv[1].x, rv[1].y, rv[1].z, rv[1].w};
      const uint32_t w2[4] = {rv[2].x, rv[2].y, rv[2].z, rv[2].w}, w3[4] = {rv[3].x, rv[3].y, rv[3].z, rv[3].w};
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        uint2 even, odd;   // d_head rows 2jj and 2jj+1 of the chunk, keys 4kg..4kg+3
        even.x = (w0[jj] & 0xffffu) | (w1[jj] << 16);
        even.y = (w2[jj] & 0xffffu) | (w3[jj] << 16);
        odd.x = (w0[jj] >> 16) | (w1[jj] & 0xffff0000u);
        odd.y = (w2[jj] >> 16) | (w3[jj] & 0xffff0000u);
        *(uint2*)(sVt + (v_c * 8 + 2 * jj) * VP + 4 * v_kg) = even;
        *(uint2*)(sVt + (v_c * 8 + 2 * jj + 1) * VP + 4 * v_kg) = odd;
      }
    }
  };

  // m_ref is the reference point of the running sum and of O (scaled scores, log2 units).  It follows the running
  // maximum lazily: it moves only when some query of the wave exceeds it by more than 8, so p stays below 2^8 and
  // most tiles skip the rescaling of O altogether; the result is the same up to rounding.
  float m_ref = -INFINITY, l_run = 0.f;
  load_regs(0);
  if (n_tiles > 0) {
    write_lds(0, 0);
    if (n_tiles > 1) load_regs(64);
  }
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int k0 = kt * 64;
    // tile kt is in place for everyone, and everyone has left tile kt-1, whose buffer tile kt+1 takes over
    __syncthreads();
    if (kt + 1 < n_tiles) {
      write_lds((kt + 1) & 1, k0 + 64);
      if (kt + 2 < n_tiles) load_regs(k0 + 128);
    }
    // a wave whose 32 queries all precede this tile has nothing to add (causal)
    if (causal && k0 > q_blk + wave * 32 + 31) continue;
    const uint4* sK = sK2[kt & 1];
    const uint16_t* sVt = sVt2[kt & 1];

    // S^T tile: 64 keys x 32 queries per wave
    f32x16 accS[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int r = 0; r < 16; ++r) accS[ks][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int r = ks * 32 + lr, c = kk * 2 + g;
        const int sw = (CPR == 8) ? (c ^ ((r >> 1) & 7)) : (c ^ (r & 15));
        accS[ks] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(sK[r * CPR + sw]), fq[kk], accS[ks], 0, 0, 0);
      }
    // mask (only the tiles that touch the diagonal or the end of the sequence), maximum of the raw scores
    const bool need_mask = (k0 + 63 >= S) || (causal && k0 + 63 > q_blk + wave * 32);
    if (need_mask) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + ks * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
          if (key >= S || (causal && key > q_row)) accS[ks][r] = -INFINITY;
        }
    }
    float mx = fmaxf(accS[0][0], accS[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(fmaxf(mx, accS[0][r]), accS[1][r]);   // one three-input max each
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2e;
    if (__any(mx > m_ref + 8.0f)) {   // also the first tile (m_ref = -inf)
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);   // m_ref = -inf -> 0
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[i][r] *= alpha;
      m_ref = m_new;
    }
    const float neg_m = (m_ref == -INFINITY) ? 0.f : -m_ref;
    float ps = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(accS[ks][r], scale_log2e, neg_m));
        accS[ks][r] = p;
        ps += p;
      }
    ps += __shfl_xor(ps, 32, 64);
    l_run += ps;

    // O^T += V^T P^T.  K step i covers keys 16i..16i+15; in operand slot (g, t) sits key
    // 16i + 8*(t/4) + 4g + t%4, which is register 8*(i%2) + t of accS[i/2].
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x8 fp;
#pragma unroll
      for (int t = 0; t < 8; ++t) fp[t] = (__bf16)accS[i >> 1][8 * (i & 1) + t];
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const uint16_t* vr = sVt + (dt * 32 + lr) * VP + 16 * i + 4 * g;
        const uint2 lo = *(const uint2*)vr;
        const uint2 hi = *(const uint2*)(vr + 8);
        const uint4 fv = make_uint4(lo.x, lo.y, hi.x, hi.y);
        accO[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fv), fp, accO[dt], 0, 0, 0);
      }
    }
  }

  if (q_row < S) {
    const float inv = (l_run > 0.f) ? 1.f / l_run : 0.f;
    bf16_t* orow = out + ((int64_t)b * S + q_row) * d + hd * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const float v[4] = {accO[dt][rg * 4] * inv, accO[dt][rg * 4 + 1] * inv, accO[dt][rg * 4 + 2] * inv,
                            accO[dt][rg * 4 + 3] * inv};
        store4(orow + dt * 32 + rg * 8 + g * 4, v);
      }
    if (lse && g == 0) lse[((int64_t)b * h + hd) * S + q_row] = m_ref * LN2 + __logf(l_run);
  }
}

// ------------------------------------------------------------------------------------------------
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_fwd_generic_kernel(const T* __restrict__ qkv, T* __restrict__ out,
                                                              float* __restrict__ lse, int32_t S, int32_t h,
                                                              int32_t causal, float scale) {
  constexpr int KT = 32;
  __shared__ float sK[KT][DH];
  __shared__ float sV[KT][DH];
  const int tid = threadIdx.x;
  const int b = blockIdx.z, hd = blockIdx.y;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * S * rs + hd * DH;
  const int q_row = blockIdx.x * 64 + tid;
  float q[DH], o[DH];
#pragma unroll
  for (int j = 0; j < DH; ++j) {
    q[j] = (q_row < S) ? to_f32(base[(int64_t)q_row * rs + j]) * scale : 0.f;
    o[j] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
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
    for (int r = 0; r < KT; ++r) {
      const int key = k0 + r;
      if (key >= S || (causal && key > q_row)) continue;
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < DH; ++j) s = fmaf(q[j], sK[r][j], s);
      const float m_new = fmaxf(m, s);
      const float alpha = __expf(m - m_new);
      const float p = __expf(s - m_new);
      l = l * alpha + p;
#pragma unroll
      for (int j = 0; j < DH; ++j) o[j] = o[j] * alpha + p * sV[r][j];
      m = m_new;
    }
  }
  if (q_row < S) {
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    T* orow = out + ((int64_t)b * S + q_row) * d + hd * DH;
#pragma unroll
    for (int j = 0; j < DH; ++j) orow[j] = from_f32<T>(o[j] * inv);
    if (lse) lse[((int64_t)b * h + hd) * S + q_row] = m + __logf(l);
  }
}

template <typename T>
hipError_t launch_generic(const void* qkv, void* out, float* lse, int32_t B, int32_t S, int32_t h, int32_t dh,
                          int32_t causal, hipStream_t st) {
  const dim3 grid((unsigned)((S + 63) / 64), (unsigned)h, (unsigned)B), block(64);
  const float scale = 1.0f / sqrtf((float)dh);
#define PF_ATT(D)                                                                                             \
  hipLaunchKernelGGL((attn_fwd_generic_kernel<T, D>), grid, block, 0, st, (const T*)qkv, (T*)out, lse, S, h, \
                     causal, scale)
  switch (dh) {
    case 8: PF_ATT(8); break;
    case 16: PF_ATT(16); break;
    case 32: PF_ATT(32); break;
    case 64: PF_ATT(64); break;
    case 128: PF_ATT(128); break;
    default: return hipErrorInvalidValue;
  }
#undef PF_ATT
  return hipGetLastError();
}

}  // namespace

hipError_t attention_fwd(int32_t dtype, const void* qkv, void* out, float* lse, int32_t B, int32_t S, int32_t h,
                         int32_t dh, int32_t causal, hipStream_t stream) {
  if (B <= 0 || S <= 0 || h <= 0 || B > 65535 || h > 65535) return hipErrorInvalidValue;
  if (dtype == PF_DTYPE_BF16_ && (dh == 64 || dh == 128)) {
    const int64_t nq = (S + 127) / 128, n_wg = nq * h * B;
    if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)n_wg), block(256);
    const float sl = LOG2E / sqrtf((float)dh);
    if (dh == 64)
      hipLaunchKernelGGL(attn_fwd_bf16_kernel<64>, grid, block, 0, stream, (const bf16_t*)qkv, (bf16_t*)out, lse, S,
                         h, causal, sl, (int32_t)nq, (int32_t)n_wg);
    else
      hipLaunchKernelGGL(attn_fwd_bf16_kernel<128>, grid, block, 0, stream, (const bf16_t*)qkv, (bf16_t*)out, lse, S,
                         h, causal, sl, (int32_t)nq, (int32_t)n_wg);
    return hipGetLastError();
  }
  if (dtype == PF_DTYPE_BF16_) return launch_generic<bf16_t>(qkv, out, lse, B, S, h, dh, causal, stream);
  return launch_generic<float>(qkv, out, lse, B, S, h, dh, causal, stream);
}

}  // namespace pf
