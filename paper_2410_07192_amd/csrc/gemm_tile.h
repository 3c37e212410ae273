// Tiled bf16 GEMM kernel for gfx950 (template) and its launcher; see gemm.hip for the overview.  Included by
// gemm.hip (dispatch) and by the gemm_inst_*.hip files, each of which instantiates some epilogue combinations so that
// they compile in parallel.
#pragma once

#include "pf_kernels.h"
#include "pf_device.h"

#include <type_traits>

namespace pf {
namespace gemm {


struct EpiDev {
  const void* bias;
  const void* resid;
  const void* dact_in;
  void* preact_out;
  int32_t gelu, accumulate;
  float scale;
};

// Epilogue for 4 consecutive columns n0..n0+3 of row m.  T = storage type of bias / resid / aux,
// OutT = type of C.  The vector form needs n0+3 < N and N % 4 == 0; the scalar form checks every
// element.
template <typename T, typename OutT>
__device__ __forceinline__ void epilogue4_vec(float v[4], int64_t m, int64_t n0, int64_t N, OutT* C,
                                              const EpiDev& ep) {
  const int64_t off = m * N + n0;
  const T* bias = (const T*)ep.bias;
  const T* resid = (const T*)ep.resid;
  const T* dact = (const T*)ep.dact_in;
  T* pre = (T*)ep.preact_out;
  float t[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] *= ep.scale;
  if (bias) {
    load4(bias + n0, t);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += t[j];
  }
  if (pre) store4(pre + off, v);
  if (ep.gelu) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = gelu_as<T>(v[j]);
  }
  if (dact) {
    load4(dact + off, t);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] *= gelu_grad_f(t[j]);
  }
  if (resid) {
    load4(resid + off, t);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += t[j];
  }
  if (ep.accumulate) {
    load4(C + off, t);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += t[j];
  }
  store4(C + off, v);
}

template <typename T, typename OutT>
__device__ __forceinline__ void epilogue4_scalar(float v[4], int64_t m, int64_t n0, int64_t M, int64_t N, OutT* C,
                                                 const EpiDev& ep) {
  if (m >= M) return;
  const int64_t off = m * N + n0;
  const T* bias = (const T*)ep.bias;
  const T* resid = (const T*)ep.resid;
  const T* dact = (const T*)ep.dact_in;
  T* pre = (T*)ep.preact_out;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (n0 + j < N) {
      float x = v[j] * ep.scale;
      if (bias) x += to_f32(bias[n0 + j]);
      if (pre) pre[off + j] = from_f32<T>(x);
      if (ep.gelu) x = gelu_as<T>(x);
      if (dact) x *= gelu_grad_f(to_f32(dact[off + j]));
      if (resid) x += to_f32(resid[off + j]);
      if (ep.accumulate) x += to_f32(C[off + j]);
      C[off + j] = from_f32<OutT>(x);
    }
  }
}

// Epilogue features the main kernel is specialised on (so that its loads carry no branches and the
// compiler can batch them); other combinations run on the generic kernel.
enum : int { E_BIAS = 1, E_GELU = 2, E_RESID = 4, E_DACT = 8, E_PRE = 16, E_ACC = 32 };

template <int EPI, typename OutT>
__device__ __forceinline__ void epilogue4_static(float v[4], const float bias4[4], int64_t off, OutT* C,
                                                 const EpiDev& ep) {
  float t[4];
  if constexpr (EPI & E_BIAS) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += bias4[j];
  }
  if constexpr (EPI & E_PRE) store4((bf16_t*)ep.preact_out + off, v);
  if constexpr (EPI & E_GELU) {
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = gelu_bf16_f(v[j]);
  }
  if constexpr (EPI & E_DACT) {
    load4((const bf16_t*)ep.dact_in + off, t);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] *= gelu_grad_f(t[j]);
  }
  if constexpr (EPI & E_RESID) {
    load4((const bf16_t*)ep.resid + off, t);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += t[j];
  }
  if constexpr (EPI & E_ACC) {
    load4(C + off, t);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] += t[j];
  }
  store4(C + off, v);
}

// compile-time loop: f(integral_constant<int, I>) for I in [0, N)
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}


// ------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// The LDS tables of the staged epilogues, behind the two operand stages; every workgroup builds its copy before the
// K loop, whose barriers publish it.
// GELU for bf16 results by table: h(x) = gelu(x) - max(x, 0) is bounded and vanishes at both ends; 1024 segments
// of 1/64 on [-8, 8), value and slope per segment, linear interpolation (error below 2.5e-5, a hundredth of a bf16
// ulp at 1).  The same for GELU' (between -0.13 and 1.13, 0 and 1 beyond the ends), where the saved
// pre-activation is bf16.
template <int NW, typename OutT, int EPI>
__device__ __forceinline__ void build_epilogue_tables(float2* gelu_tab) {
  constexpr bool GELU_TAB = std::is_same<OutT, bf16_t>::value && (EPI & E_GELU) && !(EPI & E_ACC) && NW >= 8;
  if constexpr (GELU_TAB) {
    for (int e = threadIdx.x; e < 1024; e += 64 * NW) {
      const float x0 = -8.0f + (float)e * (1.0f / 64.0f), x1 = x0 + 1.0f / 64.0f;
      const float h0 = gelu_f(x0) - fmaxf(x0, 0.f), h1 = gelu_f(x1) - fmaxf(x1, 0.f);
      gelu_tab[e] = make_float2(h0, h1 - h0);
    }
  }
  constexpr bool GRAD_TAB = std::is_same<OutT, bf16_t>::value && EPI == E_DACT;
  if constexpr (GRAD_TAB) {
    for (int e = threadIdx.x; e < 1024; e += 64 * NW) {
      const float x0 = -8.0f + (float)e * (1.0f / 64.0f);
      const float d0 = gelu_grad_f(x0), d1 = gelu_grad_f(x0 + 1.0f / 64.0f);
      gelu_tab[e] = make_float2(d0, d1 - d0);
    }
  }
}

// What a workgroup does with its finished accumulators: acc[a][b] is the 32x32 block at rows (wm * TM + b) * 32,
// columns (wn * TN + a) * 32 of the BM x BN tile at (m0, n0).  smem: the two operand stages (free after the K loop)
// followed by the table of build_epilogue_tables.
template <int WGM, int WGN, int TM, int TN, typename OutT, int EPI>
__device__ __forceinline__ void tile_epilogue(f32x16 (&acc)[TN][TM], uint4* smem, OutT* __restrict__ C, int64_t M,
                                              int64_t N, const EpiDev& ep, int64_t m0, int64_t n0) {
  constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32, NW = WGM * WGN;
  constexpr int STAGE = (BM + BN) * 8;
  float2* gelu_tab = (float2*)(smem + 2 * STAGE);
  auto gelu_grad_tab = [&](float x) {
    const float u = __builtin_amdgcn_fmed3f(fmaf(x, 64.0f, 512.0f), 0.0f, 1023.996f);
    const float2 e = gelu_tab[(int)u];
    return fmaf(e.y, __builtin_amdgcn_fractf(u), e.x);
  };
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int lr = lane & 31, lk = lane >> 5;
  // D[i][j]: lane holds j = lane%32 (row of C) and i = 8*(r/4) + 4*(lane/32) + r%4 (column of C).
  // Indices into acc must be compile-time constants or the accumulators leave the register file.
  const bool interior = (m0 + BM <= M) && (n0 + BN <= N) && ((N & 3) == 0);
  // Split K: the fp32 tile goes through LDS (row-major, 16-byte units XOR-swizzled by row) and is added to C with
  // hardware fp32 atomics, 64 consecutive columns of a row per wave instruction.  A lane-per-row atomic would touch 32
  // cache lines per instruction.  Only tiles whose fp32 image fits the two LDS stages split K (the launcher knows).
  if constexpr (std::is_same<OutT, float>::value && EPI == E_ACC && BM * BN * 4 <= 2 * STAGE * 16) {
    if (gridDim.y > 1) {
      float* stf = (float*)smem;
      constexpr int UNITS = BN / 4, NT = 64 * NW;
      static_for<0, TN>([&](auto a) {
        static_for<0, TM>([&](auto b) {
          const int row = (wm * TM + b) * 32 + lr;
          static_for<0, 4>([&](auto rg) {
            const int unit = ((wn * TN + a) * 32 + rg * 8 + lk * 4) / 4;
            *(float4*)(stf + row * BN + ((unit ^ (row & (UNITS - 1))) * 4)) =
                make_float4(acc[a][b][rg * 4 + 0], acc[a][b][rg * 4 + 1], acc[a][b][rg * 4 + 2], acc[a][b][rg * 4 + 3]);
          });
        });
      });
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_s_barrier();
#pragma unroll 8
      for (int i = 0; i < BM * BN / NT; ++i) {
        const int e = i * NT + tid, row = e / BN, col = e % BN;
        const float v = stf[row * BN + (((col >> 2) ^ (row & (UNITS - 1))) * 4) + (col & 3)];
        if (m0 + row < M && n0 + col < N) unsafeAtomicAdd((float*)C + (m0 + row) * N + n0 + col, v);
      }
      return;
    }
  }
  // Staged epilogue (bf16 output): bias and GELU are applied in registers, the bf16 tile goes through LDS (free
  // after the K loop; 16-byte slots XOR-swizzled by row) and leaves as 16-byte stores that cover whole rows of the
  // tile, the residual being added on the way out from equally coalesced loads.  The two training forms use the same
  // route: the pre-activation is a second tile staged and stored before the activated one, and the saved tensor whose
  // GELU' multiplies the result comes in the other way round, coalesced loads -> LDS -> the accumulator layout.
  constexpr bool STAGED = std::is_same<OutT, bf16_t>::value && !(EPI & E_ACC);
  if constexpr (STAGED) {
    static_assert(!(EPI & E_DACT) || EPI == E_DACT, "GELU' multiplies the plain product only");
    const bool aligned16 = ((N & 7) == 0) && ((((uintptr_t)C | (uintptr_t)ep.resid | (uintptr_t)ep.preact_out |
                                                 (uintptr_t)ep.dact_in) & 15) == 0);
    if (interior && aligned16 && N <= (1 << 21)) {
      constexpr int SLOTS = BN / 8, NT = 64 * NW, PER = BM * BN / 8 / NT;
      // 16-byte slot of a row, moved per row so that the lanes of a wave (32 rows, same column group) spread
      // over the banks: XOR when the slot count is a power of two, rotation otherwise
      auto swz = [](int slot, int row) {
        if constexpr ((SLOTS & (SLOTS - 1)) == 0) return slot ^ (row & (SLOTS - 1));
        else return (slot + row) % SLOTS;
      };
      uint2* st8 = (uint2*)smem;
      // Piece i of a thread on the way out (and of the residual on the way in): 16 bytes of row i * RP + r0 when the
      // threads of a workgroup cover whole rows.  The tile's corner is the base of a raw buffer, the thread's place a
      // 32-bit offset computed once, the rows of piece i a scalar offset (N <= 2^21 keeps all of it below 2^31): no
      // 64-bit vector arithmetic per piece, which is what a lone wave per SIMD has least of.
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      constexpr bool ROWWISE = NT % SLOTS == 0;
      constexpr int RP = ROWWISE ? NT / SLOTS : 1;
      const int r0 = tid / SLOTS, slot0 = tid % SLOTS;
      const int voff = (int)((r0 * N + slot0 * 8) * 2);
      auto tile_rsrc = [&](const void* p) {
        return __builtin_amdgcn_make_buffer_rsrc((void*)((const bf16_t*)p + m0 * N + n0), 0, 0x7fffffff, 0x00020000);
      };
      auto lds_at = [&](int i) {
        if constexpr (ROWWISE) {
          const int row = i * RP + r0;
          return row * SLOTS + swz(slot0, row);
        } else {
          const int q = i * NT + tid, row = q / SLOTS, slot = q % SLOTS;
          return row * SLOTS + swz(slot, row);
        }
      };
      auto piece_load = [&](__amdgpu_buffer_rsrc_t rs, const void* p, int i) -> uint4 {
        if constexpr (ROWWISE) {
          const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, (int)(i * RP * N * 2), 0);
          return make_uint4(v[0], v[1], v[2], v[3]);
        } else {
          const int q = i * NT + tid, row = q / SLOTS, slot = q % SLOTS;
          return *(const uint4*)((const bf16_t*)p + (m0 + row) * N + n0 + slot * 8);
        }
      };
      auto piece_store = [&](__amdgpu_buffer_rsrc_t rs, void* p, int i, uint4 v) {
        if constexpr (ROWWISE) {
          const u32x4 w = {v.x, v.y, v.z, v.w};
          __builtin_amdgcn_raw_buffer_store_b128(w, rs, voff, (int)(i * RP * N * 2), 0);
        } else {
          const int q = i * NT + tid, row = q / SLOTS, slot = q % SLOTS;
          *(uint4*)((bf16_t*)p + (m0 + row) * N + n0 + slot * 8) = v;
        }
      };
      if constexpr (EPI & E_DACT) {
        // tile of the saved pre-activation: eight 16-byte pieces per thread at a time (more would not fit beside
        // the accumulators), then every lane picks up the values of its own accumulator elements
        constexpr int CH = PER < 8 ? PER : 8;
#pragma unroll
        for (int i0 = 0; i0 < PER; i0 += CH) {
          uint4 t[CH];
#pragma unroll
          for (int i = 0; i < CH; ++i) {
            if (i0 + i < PER) {
              const int q = (i0 + i) * NT + tid, row = q / SLOTS, slot = q % SLOTS;
              t[i] = *(const uint4*)((const bf16_t*)ep.dact_in + (m0 + row) * N + n0 + slot * 8);
            }
          }
#pragma unroll
          for (int i = 0; i < CH; ++i) {
            if (i0 + i < PER) {
              const int q = (i0 + i) * NT + tid, row = q / SLOTS, slot = q % SLOTS;
              smem[row * SLOTS + swz(slot, row)] = t[i];
            }
          }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
        static_for<0, TN>([&](auto a) {
          static_for<0, TM>([&](auto b) {
            const int row = (wm * TM + b) * 32 + lr;
            static_for<0, 4>([&](auto rg) {
              const int slot = (wn * TN + a) * 4 + rg;
              const uint2 u = st8[row * (SLOTS * 2) + swz(slot, row) * 2 + lk];
              acc[a][b][rg * 4 + 0] *= gelu_grad_tab(bf16_bits_to_f32(u.x & 0xffffu));
              acc[a][b][rg * 4 + 1] *= gelu_grad_tab(bf16_bits_to_f32(u.x >> 16));
              acc[a][b][rg * 4 + 2] *= gelu_grad_tab(bf16_bits_to_f32(u.y & 0xffffu));
              acc[a][b][rg * 4 + 3] *= gelu_grad_tab(bf16_bits_to_f32(u.y >> 16));
            });
          });
        });
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();   // everyone has its values: the tile's place in LDS is free again
      }
      // accumulators (+ bias) (-> GELU) -> bf16 -> LDS in the swizzled row-major layout
      auto stage_tile = [&](auto with_gelu) {
        static_for<0, TN>([&](auto a) {
          float bias4[4][4] = {};
          if constexpr (EPI & E_BIAS) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg)
              load4((const bf16_t*)ep.bias + n0 + (wn * TN + a) * 32 + rg * 8 + lk * 4, bias4[rg]);
          }
          static_for<0, TM>([&](auto b) {
            const int row = (wm * TM + b) * 32 + lr;
            static_for<0, 4>([&](auto rg) {
              float v[4] = {acc[a][b][rg * 4 + 0], acc[a][b][rg * 4 + 1], acc[a][b][rg * 4 + 2],
                            acc[a][b][rg * 4 + 3]};
              if constexpr (EPI & E_BIAS) {
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] += bias4[rg][j];
              }
              if constexpr (decltype(with_gelu)::value) {
                // Eight waves: GELU from the table (9.5 VALU slots and one LDS gather per element; the second wave of
                // the SIMD covers the gather's latency).  Four waves, one per SIMD: nothing covers it, and the
                // arithmetic form (one exp2 and one reciprocal per element) is the faster one.
                if constexpr (NW >= 8) {
#pragma unroll
                  for (int j = 0; j < 4; ++j) {
                    const float u = __builtin_amdgcn_fmed3f(fmaf(v[j], 64.0f, 512.0f), 0.0f, 1023.996f);
                    const float2 e = gelu_tab[(int)u];
                    v[j] = fmaxf(v[j], 0.f) + fmaf(e.y, __builtin_amdgcn_fractf(u), e.x);
                  }
                } else {
#pragma unroll
                  for (int j = 0; j < 4; ++j) v[j] = gelu_bf16_f(v[j]);
                }
              }
              uint2 pk;
              pk.x = pack_bf16x2(v[0], v[1]);
              pk.y = pack_bf16x2(v[2], v[3]);
              const int slot = (wn * TN + a) * 4 + rg;
              st8[row * (SLOTS * 2) + swz(slot, row) * 2 + lk] = pk;
            });
          });
        });
      };
      if constexpr (EPI & E_PRE) {   // the value before the activation leaves first, the same way
        stage_tile(std::false_type{});
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
        const __amdgpu_buffer_rsrc_t prsrc = tile_rsrc(ep.preact_out);
#pragma unroll
        for (int i = 0; i < PER; ++i) piece_store(prsrc, ep.preact_out, i, smem[lds_at(i)]);
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
      }
      // the residual tile is requested first, in the layout of the final stores, so that it arrives while the
      // accumulators go through bias / GELU / LDS
      constexpr int EARLY = PER < 8 ? PER : 8;   // more would not fit beside the accumulators
      uint4 rres[(EPI & E_RESID) ? PER : 1];
      const __amdgpu_buffer_rsrc_t rrsrc = tile_rsrc((EPI & E_RESID) ? ep.resid : (const void*)C);
      if constexpr (EPI & E_RESID) {
#pragma unroll
        for (int i = 0; i < EARLY; ++i) rres[i] = piece_load(rrsrc, ep.resid, i);
      }
      stage_tile(std::integral_constant<bool, (EPI & E_GELU) != 0>{});
      if constexpr (EPI & E_RESID) {   // the accumulators are dead now: the rest of the residual tile
#pragma unroll
        for (int i = EARLY; i < PER; ++i) rres[i] = piece_load(rrsrc, ep.resid, i);
      }
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_s_barrier();
      const __amdgpu_buffer_rsrc_t crsrc = tile_rsrc(C);
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        uint4 v = smem[lds_at(i)];
        if constexpr (EPI & E_RESID) {
          const uint4 r = rres[i];
          const uint32_t vw[4] = {v.x, v.y, v.z, v.w}, rw[4] = {r.x, r.y, r.z, r.w};
          uint32_t ow[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float lo = bf16_bits_to_f32(vw[j] & 0xffffu) + bf16_bits_to_f32(rw[j] & 0xffffu);
            const float hi = bf16_bits_to_f32(vw[j] >> 16) + bf16_bits_to_f32(rw[j] >> 16);
            ow[j] = pack_bf16x2(lo, hi);
          }
          v = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        }
        piece_store(crsrc, C, i, v);
      }
      return;
    }
  }
  if (interior) {
    static_for<0, TN>([&](auto a) {
      float bias4[4][4] = {};
      if constexpr (EPI & E_BIAS) {
#pragma unroll
        for (int rg = 0; rg < 4; ++rg)
          load4((const bf16_t*)ep.bias + n0 + (wn * TN + a) * 32 + rg * 8 + lk * 4, bias4[rg]);
      }
      static_for<0, TM>([&](auto b) {
        const int64_t m = m0 + (wm * TM + b) * 32 + lr;
        static_for<0, 4>([&](auto rg) {
          const int64_t n = n0 + (wn * TN + a) * 32 + rg * 8 + lk * 4;
          float v[4] = {acc[a][b][rg * 4 + 0], acc[a][b][rg * 4 + 1], acc[a][b][rg * 4 + 2],
                        acc[a][b][rg * 4 + 3]};
          epilogue4_static<EPI, OutT>(v, bias4[rg], m * N + n, C, ep);
        });
      });
    });
  } else {
    static_for<0, TN>([&](auto a) {
      static_for<0, TM>([&](auto b) {
        const int64_t m = m0 + (wm * TM + b) * 32 + lr;
        static_for<0, 4>([&](auto rg) {
          const int64_t n = n0 + (wn * TN + a) * 32 + rg * 8 + lk * 4;
          float v[4] = {acc[a][b][rg * 4 + 0], acc[a][b][rg * 4 + 1], acc[a][b][rg * 4 + 2],
                        acc[a][b][rg * 4 + 3]};
          epilogue4_scalar<bf16_t, OutT>(v, m, n, M, N, C, ep);
        });
      });
    });
  }
}

template <int WGM, int WGN, int TM, int TN, typename OutT, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_nt_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, OutT* __restrict__ C, int64_t M, int64_t N,
    int64_t K, EpiDev ep, int32_t tiles_m, int32_t tiles_n, int32_t group_m) {
  constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32, NW = WGM * WGN;
  constexpr int GX = BM / 8, G = (BM + BN) / 8, GPW = G / NW;   // 8-row groups of 1 KB; per wave
  constexpr int STAGE = (BM + BN) * 8;                          // uint4 per LDS stage
  static_assert(G % NW == 0 && GPW <= 32, "tile / wave mismatch");
  extern __shared__ uint4 smem[];
  build_epilogue_tables<NW, OutT, EPI>((float2*)(smem + 2 * STAGE));
  const int64_t tile = xcd_contiguous(blockIdx.x, (int64_t)tiles_m * tiles_n);
  const int64_t per_group = (int64_t)group_m * tiles_n;
  const int64_t grp = tile / per_group;
  const int32_t first_m = (int32_t)(grp * group_m);
  const int32_t rows_in_group = (tiles_m - first_m < group_m) ? tiles_m - first_m : group_m;
  const int32_t tm_i = first_m + (int32_t)((tile % per_group) % rows_in_group);
  const int32_t tn_i = (int32_t)((tile % per_group) / rows_in_group);
  const int64_t m0 = (int64_t)tm_i * BM, n0 = (int64_t)tn_i * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int lr = lane & 31, lk = lane >> 5;

  // split K (accumulating fp32 epilogue only): workgroup y works on columns [y, y+1) * K / gridDim.y of both operands
  const int64_t k_len = K / gridDim.y;
  X += (int64_t)blockIdx.y * k_len;
  W += (int64_t)blockIdx.y * k_len;

  // global source of this lane for each 1 KB group the wave moves per K step
  const bf16_t* src[GPW];
#pragma unroll
  for (int i = 0; i < GPW; ++i) {
    const int g = wave + i * NW;
    const bool isx = g < GX;
    const int r = (isx ? g : g - GX) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    int64_t row = (isx ? m0 : n0) + r;
    const int64_t lim = isx ? M : N;
    if (row >= lim) row = lim - 1;
    src[i] = (isx ? X : W) + row * K + c * 8;
  }
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t)smem);
  // one 1 KB group of the stage at k0 straight into LDS stage `stage` (M0 carries the LDS address)
  auto issue1 = [&](auto ic, int stage, int64_t k0) {
    constexpr int i = decltype(ic)::value;
    const int g = wave + i * NW;
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)((stage * STAGE + g * 64) * 16));
    const bf16_t* p = src[i] + k0;
    lds_direct_load_1k(dst, p);
  };
  int offW[TN], offX[TM], swW[TN], swX[TM];
#pragma unroll
  for (int a = 0; a < TN; ++a) {
    const int r = (wn * TN + a) * 32 + lr;
    offW[a] = BM * 8 + r * 8;
    swW[a] = (r >> 1) & 7;
  }
#pragma unroll
  for (int b = 0; b < TM; ++b) {
    const int r = (wm * TM + b) * 32 + lr;
    offX[b] = r * 8;
    swX[b] = (r >> 1) & 7;
  }
  f32x16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  bf16x8 fw[2][TN], fx[2][TM];
  auto load_frags = [&](int buf, const uint4* st, int kk) {
    const int c = kk * 2 + lk;
#pragma unroll
    for (int a = 0; a < TN; ++a) fw[buf][a] = as_bf16x8(st[offW[a] + (c ^ swW[a])]);
#pragma unroll
    for (int b = 0; b < TM; ++b) fx[buf][b] = as_bf16x8(st[offX[b] + (c ^ swX[b])]);
  };
  // A burst of loads right after the barrier blocks every wave at the texture-address unit (1 KB per
  // instruction at 64 B/clk) while the MFMA pipe drains; instead one load is issued before every EVERY-th
  // MFMA of the block after the barrier (index 0) and of the first SPREAD-1 blocks of the next iteration.
  constexpr int MF = TM * TN, SPREAD = 3, EVERY = SPREAD * MF / GPW;
  static_assert(EVERY >= 1 && EVERY * GPW <= SPREAD * MF, "load slots");
  auto mfma_block = [&](auto blkc, auto bufc, bool do_load, int stage, int64_t k0) {
    constexpr int blk = decltype(blkc)::value, buf = decltype(bufc)::value;
    static_for<0, MF>([&](auto mi) {
      constexpr int g = blk * MF + mi;
      if constexpr (blk < SPREAD && g % EVERY == 0 && g / EVERY < GPW) {
        if (do_load) issue1(std::integral_constant<int, g / EVERY>{}, stage, k0);
      }
      constexpr int a = mi / TM, b = mi % TM;
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][a], fx[buf][b], acc[a][b], 0, 0, 0);
    });
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;

  const int64_t nk = k_len / 64;
  // prologue: stage 0 completely; of stage 1 the share the block after a barrier issues
  static_for<0, GPW>([&](auto i) { issue1(i, 0, 0); });
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  if (nk > 1) {
    static_for<0, MF>([&](auto mi) {
      if constexpr (mi % EVERY == 0 && mi / EVERY < GPW) issue1(std::integral_constant<int, mi / EVERY>{}, 1, 64);
    });
  }
  load_frags(0, smem, 0);
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int cur = (int)(kt & 1);
    const uint4* sc = smem + cur * STAGE;
    const uint4* sn = smem + (cur ^ 1) * STAGE;
    const bool more1 = kt + 1 < nk, more2 = kt + 2 < nk;
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): fragments fetched during the previous MFMA block
    load_frags(1, sc, 1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_block(I1{}, I0{}, more1, cur ^ 1, (kt + 1) * 64);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(0, sc, 2);
    __builtin_amdgcn_sched_barrier(0);
    mfma_block(I2{}, I1{}, more1, cur ^ 1, (kt + 1) * 64);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(1, sc, 3);
    __builtin_amdgcn_sched_barrier(0);
    mfma_block(I3{}, I0{}, more1, cur ^ 1, (kt + 1) * 64);
    __builtin_amdgcn_sched_barrier(0);
    // every wave holds the last fragments of this stage in registers and the next stage has landed
    __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    if (more1) load_frags(0, sn, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_block(I0{}, I1{}, more2, cur, (kt + 2) * 64);   // stage `cur` is free: start refilling it
    __builtin_amdgcn_sched_barrier(0);
  }

  tile_epilogue<WGM, WGN, TM, TN, OutT, EPI>(acc, smem, C, M, N, ep, m0, n0);
}

// The 256x256 tile on FOUR waves (one per SIMD, wave tile 128x128, accumulators in 256 registers): per K step the
// fragment reads take 128 KB out of LDS instead of the 192 KB the eight-wave form reads, and operands travel
// global -> registers -> LDS with every load in flight for a whole K step.  A wave moves sixteen 1 KB groups per step;
// slot i of a step writes the group that was loaded into register quad i one step earlier to the LDS stage that was
// freed by the previous barrier, and then reuses the quad for the load of the stage after next: sixty-four registers
// hold one stage in flight, the memory pipeline never drains, and the one barrier of a step (in the middle of the
// last MFMA block, so that queued MFMAs cover it) both publishes the next stage and frees the current one.
// Plain loads and stores: the compiler derives the vmcnt / lgkmcnt waits; the scheduling fences keep its order.
template <typename OutT, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_nt_w4_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, OutT* __restrict__ C, int64_t M, int64_t N,
    int64_t K, EpiDev ep, int32_t tiles_m, int32_t tiles_n, int32_t group_m) {
  constexpr int WGM = 2, WGN = 2, TM = 4, TN = 4;
  constexpr int BM = 256, BN = 256, NW = 4;
  constexpr int GX = BM / 8, G = (BM + BN) / 8, GPW = G / NW;   // 8-row groups of 1 KB; sixteen per wave
  constexpr int STAGE = (BM + BN) * 8;                          // uint4 per LDS stage
  extern __shared__ uint4 smem[];
  build_epilogue_tables<NW, OutT, EPI>((float2*)(smem + 2 * STAGE));

  const int64_t tile = xcd_contiguous(blockIdx.x, (int64_t)tiles_m * tiles_n);
  const int64_t per_group = (int64_t)group_m * tiles_n;
  const int64_t grp = tile / per_group;
  const int32_t first_m = (int32_t)(grp * group_m);
  const int32_t rows_in_group = (tiles_m - first_m < group_m) ? tiles_m - first_m : group_m;
  const int32_t tm_i = first_m + (int32_t)((tile % per_group) % rows_in_group);
  const int32_t tn_i = (int32_t)((tile % per_group) / rows_in_group);
  const int64_t m0 = (int64_t)tm_i * BM, n0 = (int64_t)tn_i * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int lr = lane & 31, lk = lane >> 5;

  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a first-class vector: a struct-typed quad would live in private memory
  // Global source of this lane for each group: a 32-bit byte offset from the tile's first row (rows past the end are
  // clamped: their products are never stored), added by the load instruction itself to a wave-uniform base that
  // advances by one K step; no vector arithmetic per load.  Groups 0..7 of a wave are rows of X, 8..15 rows of W.
  static_assert(GX == 8 * NW, "a wave's first eight groups are X rows");
  uint32_t off[GPW];
#pragma unroll
  for (int i = 0; i < GPW; ++i) {
    const int g = wave + i * NW;
    const bool isx = i < GPW / 2;
    const int r = (isx ? g : g - GX) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    const int64_t last = (isx ? M - m0 : N - n0) - 1;   // last valid row of the tile
    const int64_t row = r <= last ? r : last;
    off[i] = (uint32_t)((row * K + c * 8) * 2);
  }
  // Buffer loads: the tile's first row is the base of a raw buffer (no stride, no bounds to speak of: every offset
  // stays below 2^31), the lane's offset a 32-bit register, the K step a scalar offset.
  const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(X + m0 * K), 0, 0x7fffffff, 0x00020000);
  const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(W + n0 * K), 0, 0x7fffffff, 0x00020000);
  auto gload = [&](auto ic, int64_t k0) {
    constexpr int i = decltype(ic)::value;
    return __builtin_amdgcn_raw_buffer_load_b128(i < GPW / 2 ? xrsrc : wrsrc, (int)off[i], (int)(k0 * 2), 0);
  };
  const int wro = wave * 64 + lane;   // group g of a stage starts at uint4 index g * 64: this lane's place in group `wave`
  // Fragment addresses without arithmetic in the loop.  Row r of a stage holds its 16-byte chunk c at position
  // c ^ (r / 2) % 8, and the rows a lane reads are 32 apart, so every fragment of a lane has the same swizzle: the
  // chunk of slice kk sits at ((kk ^ s1) * 2 + l0) with s1 and l0 fixed per lane.  One address per stage, operand and
  // slice (sixteen registers); the 32-row blocks and nothing else go into the instructions' immediate offsets.
  const uint4* fx_at[2][4];
  const uint4* fw_at[2][4];
  {
    const int sw = (lr >> 1) & 7, s1 = sw >> 1, l0 = lk ^ (sw & 1);
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int chunk = (kk ^ s1) * 2 + l0;
        fx_at[st][kk] = smem + st * STAGE + ((wm * TM) * 32 + lr) * 8 + chunk;
        fw_at[st][kk] = smem + st * STAGE + BM * 8 + ((wn * TN) * 32 + lr) * 8 + chunk;
      }
  }
  f32x16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  bf16x8 fw[2][TN], fx[2][TM];
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;
  // fragment j of a 16-wide slice, in the order the MFMAs first need them: W block 0, the four X blocks, W blocks 1..3
  auto load_frag = [&](auto bufc, auto jc, auto stc, auto kkc) {
    constexpr int buf = decltype(bufc)::value, j = decltype(jc)::value, st = decltype(stc)::value, kk = decltype(kkc)::value;
    if constexpr (j == 0) fw[buf][0] = as_bf16x8(fw_at[st][kk][0]);
    else if constexpr (j <= 4) fx[buf][j - 1] = as_bf16x8(fx_at[st][kk][(j - 1) * 256]);
    else fw[buf][j - 4] = as_bf16x8(fw_at[st][kk][(j - 4) * 256]);
  };
  u32x4 R[GPW];
  constexpr int MF = TM * TN;   // 16 MFMAs per 16-wide slice of the K step
  // One 16-wide slice KK of a K step: sixteen MFMAs on fragment buffer KK & 1, each preceded by exactly ONE memory
  // instruction, so that none of them has to wait for an issue slot behind another (a wave issues in order, and with
  // one wave per SIMD whatever stalls it stalls the MFMA pipe).  Slices 0..2: eight fragment reads for the next slice,
  // then four times {write register quad q to the next stage, reload it for the stage after next}.  Slice 3: the last
  // four writes and reloads first, the barrier behind the eighth MFMA, then the first fragments of the next stage.
  // WR: stage kt + 1 exists (its groups wait in R); LD: stage kt + 2 exists.
  auto slice = [&](auto kkc, auto wrc, auto ldc, auto curc, int64_t k_next2) {
    constexpr int KK = decltype(kkc)::value, buf = KK & 1, nbuf = buf ^ 1, CUR = decltype(curc)::value;
    uint4* const sn = smem + (CUR ^ 1) * STAGE;
    constexpr bool WR = decltype(wrc)::value, LD = decltype(ldc)::value;
    static_for<0, MF>([&](auto mi) {
      // One wait per group instead of one per use (the compiler, which still places every wait that is needed,
      // drops its own where these make them redundant): all eight fragments of this slice, read eight to sixteen
      // instructions ago with four LDS stores behind them, at the slice's first MFMA; the four register quads about
      // to be stored, loaded a K step ago with twelve younger loads behind them, at the first store.
      if constexpr (mi == 0 && KK > 0) __builtin_amdgcn_s_waitcnt(0xc47f);                                   // lgkmcnt(4)
      if constexpr (WR && LD && ((KK < 3 && mi == 8) || (KK == 3 && mi == 0))) __builtin_amdgcn_s_waitcnt(0x0f7c);   // vmcnt(12)
      if constexpr (KK < 3) {
        if constexpr (mi < 8) {
          load_frag(std::integral_constant<int, nbuf>{}, mi, curc, std::integral_constant<int, (KK + 1) & 3>{});
        } else {
          constexpr int q = 4 * KK + (mi - 8) / 2;
          if constexpr ((mi & 1) == 0) {
            if constexpr (WR) *(u32x4*)(sn + wro + q * NW * 64) = R[q];
          } else {
            if constexpr (LD) R[q] = gload(std::integral_constant<int, q>{}, k_next2);
          }
        }
      } else {
        if constexpr (mi < 4) {
          if constexpr (WR) *(u32x4*)(sn + wro + (12 + mi) * NW * 64) = R[12 + mi];
        } else if constexpr (mi < 8) {
          if constexpr (LD) R[8 + mi] = gload(std::integral_constant<int, 8 + mi>{}, k_next2);
        } else {
          if constexpr (mi == 8) {
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): my LDS writes are done, my last fragments are in registers
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
          }
          if constexpr (WR) load_frag(std::integral_constant<int, nbuf>{}, std::integral_constant<int, mi - 8>{}, std::integral_constant<int, CUR ^ 1>{}, I0{});
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      constexpr int a = mi / TM, b = mi % TM;
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][a], fx[buf][b], acc[a][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  // The stage is a compile-time constant (its addresses are picked from registers, not computed), so even and odd K
  // steps are separate instantiations.  Step kt works on stage (kt + nk) % 2: the last step is then always on stage
  // 1 and the one before it on stage 0 whatever nk is, and only the very first step of an odd nk stands alone.
  auto step = [&](auto wrc, auto ldc, auto curc, int64_t k_next2) {
    slice(I0{}, wrc, ldc, curc, k_next2);
    slice(I1{}, wrc, ldc, curc, k_next2);
    slice(I2{}, wrc, ldc, curc, k_next2);
    slice(I3{}, wrc, ldc, curc, k_next2);
  };

  const int64_t nk = K / 64;
  const int s0 = (int)(nk & 1);
  // prologue: K step 0 through the registers into its stage, step 1 into the registers, the first fragments
  static_for<0, GPW>([&](auto i) { R[i] = gload(i, 0); });
  static_for<0, GPW>([&](auto i) { *(u32x4*)(smem + s0 * STAGE + wro + i * NW * 64) = R[i]; });
  if (nk > 1) static_for<0, GPW>([&](auto i) { R[i] = gload(i, 64); });
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __builtin_amdgcn_s_barrier();
  if (s0) static_for<0, 8>([&](auto j) { load_frag(I0{}, j, I1{}, I0{}); });
  else static_for<0, 8>([&](auto j) { load_frag(I0{}, j, I0{}, I0{}); });
  int64_t kt = 0;
  if (nk >= 3 && s0) {
    step(std::true_type{}, std::true_type{}, I1{}, 2 * 64);
    kt = 1;
  }
  for (; kt + 2 < nk; kt += 2) {
    step(std::true_type{}, std::true_type{}, I0{}, (kt + 2) * 64);
    step(std::true_type{}, std::true_type{}, I1{}, (kt + 3) * 64);
  }
  if (nk >= 2) step(std::true_type{}, std::false_type{}, I0{}, 0);
  step(std::false_type{}, std::false_type{}, I1{}, 0);

  tile_epilogue<WGM, WGN, TM, TN, OutT, EPI>(acc, smem, C, M, N, ep, m0, n0);
}

template <typename OutT, typename Kern>
hipError_t launch_tiles(Kern kern, int BM, int BN, int threads, bool* attr_set, const void* X, const void* W, void* C,
                        int64_t M, int64_t N, int64_t K, const EpiDev& ep, int32_t splits, hipStream_t stream) {
  const int64_t tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const size_t lds = (size_t)2 * (BM + BN) * 8 * sizeof(uint4) + 8192;   // two stages + the GELU table
  if (!*attr_set) {   // raise the dynamic-LDS limit once per instantiation
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    *attr_set = true;
  }
  const int32_t group_m = 8;
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n), (unsigned)splits), dim3(threads), lds, stream, (const bf16_t*)X,
                     (const bf16_t*)W, (OutT*)C, M, N, K, ep,
                     (int32_t)tiles_m, (int32_t)tiles_n, group_m);
  return hipGetLastError();
}

// Main kernel for one epilogue combination.  Tile shapes: 256x256 (the four-wave kernel above, wave tile 128x128),
// 256x192 (8 waves as 4x2, wave tile 64x96), both one workgroup per CU, and 128x128 (4 waves, two workgroups per CU).
// A launch takes ceil(workgroups / resident workgroups) rounds of (K steps + a fixed cost of about 4 steps); the
// shape with the least estimated time rounds x steps x area in flight per CU / efficiency is taken.  Efficiencies
// are measured on MI355X relative to the 256x256 tile (0.96 and 0.85); a shape that leaves partial tiles along N
// pays for their slower epilogue.  E.g. N = 768 or 2304 fills whole rounds with 192-wide tiles but wastes a quarter
// of the last round with 256-wide ones, and a 8192 x 1024 result gives every CU work only with the small tile.
// Accumulating fp32 launches (weight gradients: small M x N, K = all tokens) may split K over up to 8 workgroups
// per 128x128 tile while that fills idle CUs and leaves each >= 8 K steps; the slices add into C with fp32 atomics
// (order-dependent in the last bits, like the other atomic reductions over tokens).  Those atomics go at about
// 1.5 TB/s on MI355X, far below plain stores, so the estimate charges every slice for its tile: two slices usually
// pay, eight rarely do.  (256-wide tiles with split K were measured too: their atomic bursts at the end of the one
// round are not hidden by anything and they lose to the small tile on every weight-gradient shape tried.)
template <typename OutT, int EPI>
hipError_t launch_fast(const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K, const EpiDev& ep,
                       hipStream_t stream) {
  static bool attr_big = false, attr_wide = false, attr_small = false;
  struct Shape { int bm, bn, resident, eff100; } const shapes[3] = {{256, 256, 256, 100}, {256, 192, 256, 104},
                                                                      {128, 128, 512, 118}};
  int best = 0, best_splits = 1;
  int64_t best_cost = -1;
  for (int i = 0; i < 3; ++i) {
    const Shape& sh = shapes[i];
    const int64_t tiles = ((M + sh.bm - 1) / sh.bm) * ((N + sh.bn - 1) / sh.bn);
    int max_splits = 1;
    if constexpr (std::is_same<OutT, float>::value && EPI == E_ACC) max_splits = (i == 2) ? 8 : 1;
    for (int splits = 1; splits <= max_splits; splits *= 2) {
      // a slice keeps >= 8 K steps, and splitting only fills CUs that would otherwise idle
      if (splits > 1 && (K % (128 * splits) != 0 || K / (128 * splits) < 8 || tiles * splits > sh.resident)) break;
      const int64_t wgs = tiles * splits;
      const int64_t rounds = (wgs + sh.resident - 1) / sh.resident;
      const int64_t steps = K / (64 * splits) + 4;
      // area in flight per CU x relative cost: a 128x128 workgroup that has its CU to itself runs 1.4x as fast as
      // one of a pair, not twice
      int64_t per_step = (int64_t)(sh.resident / 256) * sh.bm * sh.bn * sh.eff100;
      if (i == 2 && wgs <= 256) per_step = (int64_t)sh.bm * sh.bn * 165;
      int64_t cost = rounds * steps * per_step;
      if (N % sh.bn) cost += cost * 3 / 10;
      // every slice adds its whole fp32 tile with atomics: about 0.67 us per MiB, in the units of this estimate
      if (splits > 1) cost += M * N * splits * 10;
      if (best_cost < 0 || cost < best_cost) {
        best_cost = cost;
        best = i;
        best_splits = splits;
      }
    }
  }
  if (best == 0)
    return launch_tiles<OutT>(gemm_bf16_nt_w4_kernel<OutT, EPI>, 256, 256, 256, &attr_big, X, W, C, M, N, K, ep, 1, stream);
  if (best == 1)
    return launch_tiles<OutT>(gemm_bf16_nt_kernel<4, 2, 2, 3, OutT, EPI>, 256, 192, 512, &attr_wide, X, W, C, M, N, K, ep,
                              1, stream);
  return launch_tiles<OutT>(gemm_bf16_nt_kernel<2, 2, 2, 2, OutT, EPI>, 128, 128, 256, &attr_small, X, W, C, M, N, K, ep,
                            best_splits, stream);
}

}  // namespace gemm
}  // namespace pf
