// Attention forward for gfx950.
//
// bf16, d_head 64 or 128: flash-style kernel.  A workgroup of 8 (d_head 64) or 4 (d_head 128) waves owns 256 or
// 128 queries of one (batch, head); each wave owns 32 of them and walks the keys in tiles of 64 staged in LDS.  The
// kernel computes S^T = K Q^T with the 32x32x16 bf16 MFMA (K tile rows are the "A" operand, the
// wave's Q rows the "B" operand, kept in registers), so that a lane holds 32 of the 64 scores of ONE
// query: the running sum is kept per lane, the rescale factor is a per-lane scalar, and the two lanes of a
// query (lane ^ 32) exchange values only when the reference point of the softmax moves and after the last tile.  The probabilities, already in the "B" operand layout, then feed
// O^T = V^T P^T.  K and V tiles go global -> LDS directly, row-major as they lie in memory; the V^T "A" operand
// comes out of the row-major V tile through the transposing LDS load (ds_read_b64_tr_b16), two per fragment.
//
// Generic path (fp32, or any d_head in {8,16,32,64,128}): one thread per query, keys staged in LDS,
// online softmax key by key.  Used for the small fp32 parity workload and odd head sizes.
#include "pf_kernels.h"
#include "pf_device.h"


namespace pf {
namespace {

constexpr float LOG2E = 1.4426950408889634f;

// Compute units of the current device, rounded down to a multiple of 8 (the XCDs); cached per device.
inline int compute_units() {
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
    cached[dev] = n & ~7;
  }
  return cached[dev];
}
constexpr float LN2 = 0.6931471805599453f;

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(3))) char* lds_char_ptr;

// ------------------------------------------------------------------------------------------------
// PERSIST: the grid holds as many workgroups as the CUs keep resident, and each walks the units (batch, head, block
// of QB queries) v = blockIdx.x, blockIdx.x + gridDim.x, ...  A workgroup that starts from scratch spends several
// microseconds before its first MFMA (launch, kernel arguments, Q, the first K/V tile), as long as four to eight
// tiles take; here the next unit's first tile is copied into the free LDS buffer during the current unit's last tile
// and its Q fragments are requested before the current unit's results are stored, and a workgroup's units can be
// chosen so that their lengths even out.  Otherwise one workgroup per unit (the launcher says which form pays where).
template <int DH, int NW, bool PERSIST>
__global__ __launch_bounds__(64 * NW, (DH == 64 ? 16 : 8) / NW) void attn_fwd_bf16_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out,
                                                            float* __restrict__ lse, int32_t S, int32_t h,
                                                            int32_t causal, float scale_log2e, int32_t nq,
                                                            int32_t n_units, int32_t flip) {
  constexpr int CPR = DH / 8;        // 16-byte chunks per row
  constexpr int KS = DH / 16;        // MFMA K steps over d_head
  constexpr int DT = DH / 32;        // 32-row tiles of O^T
  constexpr int ROWB = DH * 2;       // bytes per K or V row
  constexpr int TILE = 64 * ROWB;    // bytes per tile of 64 keys
  constexpr int NI = TILE / 1024;    // wave-wide copies (1 KB each) per tile
  constexpr int RPI = 1024 / ROWB;   // rows per copy
  constexpr int PER = 2 * NI / NW;   // copies per wave per (K, V) tile pair
  constexpr int QB = 32 * NW;        // queries per workgroup
  // two buffers of (K tile | V tile), both row-major as in memory, 16-byte chunks swizzled within a row
  __shared__ __align__(16) char smem[2 * 2 * TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, g = lane >> 5;
  const int d = h * DH;
  const int64_t rs = 3 * (int64_t)d;                       // row stride of qkv
  // Rows are addressed by a 32-bit row number times the row stride, clamped to the last row of the sequence, so
  // that no load sits in a branch: a clamped row repeats the last row of the sequence, which the tile holds anyway,
  // and the scores of the keys past the end are masked, so their probabilities are 0.
  const uint32_t rs32 = (uint32_t)rs;

  // Unit v of round k = v / gridDim.x.  Workgroup ids are dealt round-robin to the 8 XCDs and the grid is a multiple
  // of 8, so a workgroup stays on its XCD; xcd_contiguous gives each XCD a contiguous range of units, the query
  // blocks of one head run on one XCD at about the same time and its L2 serves their repeated reads of that head's
  // K and V.  Causal: a block's work grows with its position.  Within a round the blocks of a head are handed out
  // longest first.  flip 1 (persistent; every round's units are whole heads, the launcher checks): odd rounds hand
  // them out in the opposite order, so that a workgroup that drew a long block in one round draws a short one in
  // the next.  flip 2 (one round, all units resident at once; the two halves of an XCD's range are whole heads):
  // the second half is handed out in the opposite order, so that the two workgroups that share a CU (ids 32 x 8
  // apart on the same XCD) are a long and a short block.
  struct Unit { int b, hd, q_blk; };
  auto unit_of = [&](int v) {
    const int u = (int)xcd_contiguous(v, n_units);
    int pos = u % nq;
    if (flip == 1 && ((v / (int)gridDim.x) & 1)) pos = nq - 1 - pos;
    if (flip == 2 && (v >> 3) >= (n_units >> 4)) pos = nq - 1 - pos;
    Unit r;
    r.b = u / (nq * h);
    r.hd = (u / nq) % h;
    r.q_blk = (causal ? nq - 1 - pos : pos) * QB;
    return r;
  };
  auto base_of = [&](const Unit& u) { return qkv + (int64_t)u.b * S * rs + u.hd * DH; };

  // Swizzles (XOR on the 16-byte chunk index of a row).  K is read as the MFMA "A" operand, one 16-byte chunk per
  // lane, 32 consecutive rows per half-wave: rows are spread over the banks by (row / 2) % 8 (d_head 64: two rows
  // per 256 bytes) or row % 16.  V is read through the transposing LDS load, where 16 lanes fetch a 4-key x
  // 32-byte block: the 32-byte pairs of the four rows must fall on different banks, so the pair index is flipped
  // by (row / 2) % 2 (d_head 64: rows r and r+1 already sit in different halves of the banks) or row % 4.
  auto swz_k = [](int r) { return CPR == 8 ? ((r >> 1) & 7) : (r & 15); };
  auto swz_v = [](int r) { return CPR == 8 ? (((r >> 1) & 1) << 1) : ((r & 3) << 1); };

  // Tile staging: global -> LDS directly, no registers in between.  One wave-wide copy moves 1 KB = RPI rows into
  // consecutive LDS bytes (lane i -> byte 16 i); which chunk of the row a lane fetches undoes the swizzle.  Copy q
  // of a tile belongs to wave q % NW; a wave's copy i (i < PER / 2: K, else V) covers rows from st_row + NW i RPI,
  // all congruent modulo the period of both swizzles, so one chunk offset per operand serves every copy.
  static_assert((NW * RPI) % 16 == 0 && NI % NW == 0, "rows of one lane's copies must share their swizzle");
  const int st_row = wave * RPI + lane / CPR;
  const int st_col_k = d + (((lane % CPR) ^ swz_k(st_row)) << 3);
  const int st_col_v = 2 * d + (((lane % CPR) ^ swz_v(st_row)) << 3);
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_ptr)smem);
  auto stage = [&](int buf, const bf16_t* base, int k0) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      constexpr int HALF = PER / 2;
      const bool is_v = i >= HALF;
      const int q = wave + NW * (i % HALF);   // copy index within the K or V tile
      const uint32_t dst =
          __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)(buf * 2 * TILE + (is_v ? TILE : 0) + q * 1024));
      int row = k0 + st_row + NW * (i % HALF) * RPI;
      row = row < S ? row : S - 1;
      const bf16_t* p = base + (uint64_t)(uint32_t)row * rs32 + (is_v ? st_col_v : st_col_k);
      lds_direct_load_1k(dst, p);
    }
  };
  bf16x8 fq[KS];
  auto load_q = [&](const bf16_t* base, int q_blk) {
    const int q_row = q_blk + wave * 32 + lr;
    const bf16_t* qp = base + (uint64_t)(uint32_t)(q_row < S ? q_row : S - 1) * rs32 + g * 8;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) fq[kk] = as_bf16x8(*(const uint4*)(qp + kk * 16));
  };

  // V^T operand of O^T += V^T P^T for K step i (keys 16 i .. 16 i + 15) and d_head block dt: lane 16 G + p points
  // at key 16 i + 8 r + 4 g + p / 4 (r = 0, 1 the two reads) and at the four d_head columns from
  // 32 dt + 16 (G % 2) + 4 (p % 4); it receives column 32 dt + lane % 32 of the four keys, which is the order the
  // probabilities have in the "B" operand registers.
  int v_off[DT];
  {
    const int pl = lane & 15, mb = (lane >> 4) & 1, row = 4 * g + (pl >> 2);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int c = dt * 4 + mb * 2 + ((pl & 3) >> 1);
      v_off[dt] = TILE + row * ROWB + ((c ^ swz_v(row)) << 4) + 8 * (pl & 1);   // swz_v(row + 8 r + 16 i) = swz_v(row)
    }
  }

  // x[lane ^ 32] without the LDS: the swap leaves (low half of x, low half of x) in one register and (high half,
  // high half) in the other; callers combine the two with a commutative operation.  (The results go through an
  // empty asm statement: the compiler otherwise folds fmaxf of the two into the first.)
  auto halves = [](float x, float& lo, float& hi) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    unsigned a = r[0], b = r[1];
    asm volatile("" : "+v"(a), "+v"(b));
    lo = __builtin_bit_cast(float, a);
    hi = __builtin_bit_cast(float, b);
  };

  int gt = 0;   // tiles staged so far by this workgroup: tile t of a unit lives in buffer (gt + t) % 2
  int v = blockIdx.x;
  Unit un = unit_of(v);
  const bf16_t* base = base_of(un);
  // The first tile's copies go out while the Q fragments are still on their way (one memory latency, not two).
  stage(0, base, 0);
  load_q(base, un.q_blk);
  for (;;) {
    const int q_blk = un.q_blk;
    const int q_row = q_blk + wave * 32 + lr;                // this lane's query
    const int vn = v + (int)gridDim.x;
    const bool more = PERSIST && vn < n_units;
    Unit un_next = un;
    if (more) un_next = unit_of(vn);
    const bf16_t* base_next = base_of(un_next);
    // The Q fragments are waited for here, once: left pending, the compiler would wait for them in every iteration
    // with a count that also holds back the copies issued just before.  After the first unit the previous unit's
    // stores are younger than these loads; a count that lets younger stores stay in flight relies on stores and
    // loads retiring in one order, so everything is waited for (the first tile's copies are needed next anyway).
    if (PERSIST) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" ::"v"(fq[kk]));

    f32x16 accO[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) accO[i][r] = 0.f;
    int n_tiles = (S + 63) / 64;
    if (causal) {
      const int last_q = (q_blk + QB - 1 < S - 1) ? q_blk + QB - 1 : S - 1;
      const int need = last_q / 64 + 1;
      if (need < n_tiles) n_tiles = need;
    }
    // m_ref is the reference point of the running sum and of O (scaled scores, log2 units).  It follows the running
    // maximum lazily: it moves only when a lane's share of a tile's row sum against it exceeds 2^7, so most tiles
    // compute no maximum and skip the rescaling of O; the result is the same up to rounding.  l_run is this lane's
    // share of the row sum (32 of every 64 keys).
    float m_ref = -INFINITY, l_run = 0.f;
    for (int kt = 0; kt < n_tiles; ++kt) {
      const int k0 = kt * 64;
      // tile kt has landed (every wave waits for its own copies, then the barrier), and everyone has left the tile
      // before it, whose buffer the next tile takes over: tile kt + 1 of this unit, or the first of the next unit
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (kt + 1 < n_tiles) stage((gt + kt + 1) & 1, base, k0 + 64);
      else if (more) stage((gt + kt + 1) & 1, base_next, 0);
      // a wave whose 32 queries all precede this tile has nothing to add (causal)
      if (!(causal && k0 > q_blk + wave * 32 + 31)) {
        const char* sKb = smem + ((gt + kt) & 1) * 2 * TILE;
        lds_char_ptr sVb = (lds_char_ptr)(lds_void_ptr)smem + ((gt + kt) & 1) * 2 * TILE;

      // S^T tile: 64 keys x 32 queries per wave; masked only in the tiles that touch the diagonal or the end of the
      // sequence
      f32x16 accS[2];
      auto scores = [&] {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int r = 0; r < 16; ++r) accS[ks][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) {
            const int r = ks * 32 + lr, c = kk * 2 + g;
            const uint4 fk = *(const uint4*)(sKb + r * ROWB + ((c ^ swz_k(r)) << 4));
            accS[ks] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fk), fq[kk], accS[ks], 0, 0, 0);
          }
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
      };
      scores();
      // The exponentials are taken against the reference point as it stands, without looking at the tile's maximum
      // first; the lane's share of the row sum tells afterwards whether that was good enough.
      const float neg_m = (m_ref == -INFINITY) ? 0.f : -m_ref;
      float ps4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          accS[ks][r] = __builtin_amdgcn_exp2f(fmaf(accS[ks][r], scale_log2e, neg_m));
          ps4[r & 3] += accS[ks][r];
        }
      float tot = (ps4[0] + ps4[1]) + (ps4[2] + ps4[3]);   // this lane's 32 of the tile's 64 keys
      // Rare path: some query of the wave has no reference point yet (first tile), or its probabilities against the
      // old one add up to more than 2^7 per lane (also inf or NaN): the scores are computed again, the reference point
      // moves to the running maximum, O and the running sum are rescaled, and the exponentials are taken against the
      // new reference point.
      if (__any(!(tot <= 128.0f) || m_ref == -INFINITY)) {
        scores();
        float mx0 = fmaxf(accS[0][0], accS[1][0]), mx1 = fmaxf(accS[0][1], accS[1][1]);   // three-input maxima
#pragma unroll
        for (int r = 2; r < 16; r += 2) {
          mx0 = fmaxf(fmaxf(mx0, accS[0][r]), accS[1][r]);
          mx1 = fmaxf(fmaxf(mx1, accS[0][r + 1]), accS[1][r + 1]);
        }
        float mlo, mhi;
        halves(fmaxf(mx0, mx1), mlo, mhi);
        const float m_new = fmaxf(m_ref, fmaxf(mlo, mhi) * scale_log2e);
        const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);   // m_ref = -inf -> 0
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) accO[i][r] *= alpha;
        m_ref = m_new;
        const float neg_m2 = (m_ref == -INFINITY) ? 0.f : -m_ref;
        tot = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            accS[ks][r] = __builtin_amdgcn_exp2f(fmaf(accS[ks][r], scale_log2e, neg_m2));
            tot += accS[ks][r];
          }
      }
      l_run += tot;   // per lane: the two halves of a query's sum meet after the last tile

      // O^T += V^T P^T.  K step i covers keys 16i..16i+15; in operand slot (g, t) sits key
      // 16i + 8*(t/4) + 4g + t%4, which is register 8*(i%2) + t of accS[i/2].
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bf16x8 fp;
#pragma unroll
        for (int t = 0; t < 8; ++t) fp[t] = (__bf16)accS[i >> 1][8 * (i & 1) + t];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          lds_char_ptr vp = sVb + v_off[dt] + 16 * i * ROWB;
          const v4s r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)vp);
          const v4s r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(vp + 8 * ROWB));
          v8s fv;
          fv[0] = r0[0]; fv[1] = r0[1]; fv[2] = r0[2]; fv[3] = r0[3];
          fv[4] = r1[0]; fv[5] = r1[1]; fv[6] = r1[2]; fv[7] = r1[3];
          accO[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fv), fp, accO[dt], 0, 0, 0);
        }
      }
      }
    }
    gt += n_tiles;
    if (more) load_q(base_next, un_next.q_blk);   // on their way while this unit's results are stored

    {
      float llo, lhi;
      halves(l_run, llo, lhi);
      l_run = llo + lhi;
    }
    if (q_row < S) {
      const float inv = (l_run > 0.f) ? 1.f / l_run : 0.f;
      bf16_t* orow = out + ((int64_t)un.b * S + q_row) * d + un.hd * DH;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const float vv[4] = {accO[dt][rg * 4] * inv, accO[dt][rg * 4 + 1] * inv, accO[dt][rg * 4 + 2] * inv,
                               accO[dt][rg * 4 + 3] * inv};
          store4(orow + dt * 32 + rg * 8 + g * 4, vv);
        }
      if (lse && g == 0) lse[((int64_t)un.b * h + un.hd) * S + q_row] = m_ref * LN2 + __logf(l_run);
    }
    if (!more) break;
    v = vn;
    un = un_next;
    base = base_next;
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
    // d_head 64: eight waves (256 queries) per workgroup share a K/V tile, which halves the copies per wave (-7 % on
    // the causal 1024-token shape, -1.5 % on 512 tokens); d_head 128 with eight is 13 % slower (one workgroup per CU)
    constexpr int NW64 = 8, NW128 = 4;
    const int qb = 32 * (dh == 64 ? NW64 : NW128);
    const int64_t nq = (S + qb - 1) / qb, n_units = nq * h * B;
    if (n_units > 0x7fffffff) return hipErrorInvalidValue;
    const float sl = LOG2E / sqrtf((float)dh);
    const dim3 block((unsigned)(2 * qb));
    // The persistent form pays for causal d_head 128 (MI355X, same box: 116 -> 89 us on 64 heads of 2048 tokens,
    // 140 -> 122 us on 256 heads of 1024): units of unequal length even out over a workgroup's rounds and the next
    // unit's first loads hide behind the current one.  With equal units (not causal) the hardware's own dispatch
    // of one workgroup per unit is 5 % faster, and with d_head 64 the persistent loop needs one register more than
    // the 128 that four waves per SIMD allow.
    const int64_t resident = 2 * (int64_t)compute_units();   // two workgroups per CU at a time (LDS)
    if (dh == 128 && causal && n_units > resident) {
      // odd rounds may hand a head's blocks out in the opposite order only if every round's share of an XCD's range
      // is whole heads: the reversal then permutes units within the round
      const int32_t flip = (n_units % (8 * nq) == 0 && (resident / 8) % nq == 0) ? 1 : 0;
      hipLaunchKernelGGL((attn_fwd_bf16_kernel<128, NW128, true>), dim3((unsigned)resident), block, 0, stream,
                         (const bf16_t*)qkv, (bf16_t*)out, lse, S, h, causal, sl, (int32_t)nq, (int32_t)n_units, flip);
    } else {
      // one round: pair long and short causal blocks on a CU where the halves of every XCD's range are whole heads
      // (MI355X, same box: 41.8 -> 33.9 us on 128 heads of 1024 tokens with d_head 64, 73.7 -> 55.7 us on 64 heads of 2048)
      const int32_t flip = (causal && nq > 1 && n_units <= resident && n_units % 16 == 0 && (n_units / 16) % nq == 0) ? 2 : 0;
      if (dh == 64)
        hipLaunchKernelGGL((attn_fwd_bf16_kernel<64, NW64, false>), dim3((unsigned)n_units), block, 0, stream,
                           (const bf16_t*)qkv, (bf16_t*)out, lse, S, h, causal, sl, (int32_t)nq, (int32_t)n_units, flip);
      else
        hipLaunchKernelGGL((attn_fwd_bf16_kernel<128, NW128, false>), dim3((unsigned)n_units), block, 0, stream,
                           (const bf16_t*)qkv, (bf16_t*)out, lse, S, h, causal, sl, (int32_t)nq, (int32_t)n_units, flip);
    }
    return hipGetLastError();
  }
  if (dtype == PF_DTYPE_BF16_) return launch_generic<bf16_t>(qkv, out, lse, B, S, h, dh, causal, stream);
  return launch_generic<float>(qkv, out, lse, B, S, h, dh, causal, stream);
}

}  // namespace pf
