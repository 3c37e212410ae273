// GEMM kernels for gfx950:  C[M,N] = epilogue( X[M,K] * W[N,K]^T ).
//
// bf16 main path (K a multiple of 64): 32x32x16 bf16 MFMA, fp32 accumulators.  A workgroup of
// WGM x WGN waves owns a (WGM*TM*32) x (WGN*TN*32) tile of C and walks K in steps of 64.
//  * Operand tiles go from global memory straight into LDS (global_load_lds, 16 bytes per lane, no
//    VGPR round trip).  A wave's 64 lanes fill 1 KB of consecutive LDS = 8 rows of 8 chunks; the XOR
//    swizzle that keeps the later MFMA operand reads free of bank conflicts is applied on the global
//    side (lane -> which chunk of the row it fetches).  Rows beyond M / N are clamped to the last
//    valid row (their products are never stored).
//  * Two LDS stages: the loads of step k+2 go into the stage that the barrier ending step k has
//    freed.  They are issued one at a time between the MFMAs of the following blocks (a burst
//    blocks every wave at the address unit) and are inline assembly so that the compiler does not
//    serialise every later LDS read behind them; vmcnt is waited by hand.
//  * Operand fragments are double buffered in registers: the 16-byte LDS reads of sub-step kk+1
//    are in flight while the MFMAs of sub-step kk issue.
//  * The weight tile is the MFMA "A" operand and the activation tile the "B" operand, so each lane
//    ends up with 4 consecutive output columns of one output row: bias / GELU are applied in
//    registers; bf16 tiles then pass through LDS and leave as 16-byte row-contiguous stores (the
//    residual is added on the way out), other epilogues store 8- or 16-byte pieces directly.
//  * Three tile shapes (256x256, 256x192, 128x128), chosen per launch by an estimate of rounds x
//    steps x area; accumulating fp32 launches may split K (gemm_tile.h).
//  * Workgroup ids are remapped so that each of the 8 XCDs (ids are dealt round-robin to them) works
//    on a contiguous range of tiles and its L2 sees each operand panel once.
// bf16 generic path (any K multiple of 8): register-staged LDS tiles, same MFMA layout.
// fp32 path (small parity workload only): plain LDS-tiled FMA kernel with the same epilogue.
#include "pf_kernels.h"
#include "gemm_tile.h"

namespace pf {
namespace gemm {

extern template hipError_t launch_fast<bf16_t, 0>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
extern template hipError_t launch_fast<bf16_t, E_BIAS>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
extern template hipError_t launch_fast<bf16_t, E_BIAS | E_GELU>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
extern template hipError_t launch_fast<bf16_t, E_BIAS | E_RESID>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
extern template hipError_t launch_fast<bf16_t, E_BIAS | E_GELU | E_PRE>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
extern template hipError_t launch_fast<bf16_t, E_DACT>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
extern template hipError_t launch_fast<float, 0>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);
extern template hipError_t launch_fast<float, E_ACC>(const void*, const void*, void*, int64_t, int64_t, int64_t, const EpiDev&, hipStream_t);

}  // namespace gemm

namespace {

using namespace gemm;

// ------------------------------------------------------------------------------------------------
template <int WGM, int WGN, int TM, int TN, typename OutT>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_nt_generic_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, OutT* __restrict__ C, int64_t M, int64_t N,
    int64_t K, EpiDev ep, int32_t tiles_m, int32_t tiles_n, int32_t group_m) {
  constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32, NT = 64 * WGM * WGN;
  constexpr int XCH = BM * 8 / NT, WCH = BN * 8 / NT;   // 16-byte chunks per thread per K step
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile / thread mismatch");
  extern __shared__ uint4 smem[];
  // buffer b: X tile at smem + b*(BM+BN)*8, W tile right after it

  // tile coordinates: contiguous range per XCD, grouped so `group_m` row tiles share the sweep over N
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

  uint4 rx[XCH], rw[WCH];
  auto load_global = [&](int64_t k0) {
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
      const int q = tid + i * NT, r = q >> 3, c = q & 7;
      const int64_t gm = m0 + r, gk = k0 + c * 8;
      rx[i] = (gm < M && gk < K) ? *(const uint4*)(X + gm * K + gk) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < WCH; ++i) {
      const int q = tid + i * NT, r = q >> 3, c = q & 7;
      const int64_t gn = n0 + r, gk = k0 + c * 8;
      rw[i] = (gn < N && gk < K) ? *(const uint4*)(W + gn * K + gk) : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XCH; ++i) {
      const int q = tid + i * NT, r = q >> 3, c = q & 7;
      smem[buf * (BM + BN) * 8 + r * 8 + (c ^ ((r >> 1) & 7))] = rx[i];
    }
#pragma unroll
    for (int i = 0; i < WCH; ++i) {
      const int q = tid + i * NT, r = q >> 3, c = q & 7;
      smem[buf * (BM + BN) * 8 + BM * 8 + r * 8 + (c ^ ((r >> 1) & 7))] = rw[i];
    }
  };

  f32x16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  const int64_t nk = (K + 63) / 64;
  load_global(0);
  store_lds(0);
  __syncthreads();
  const int lr = lane & 31, lk = lane >> 5;
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int cur = (int)(kt & 1);
    const uint4* sXc = smem + cur * (BM + BN) * 8;
    const uint4* sWc = sXc + BM * 8;
    if (kt + 1 < nk) load_global((kt + 1) * 64);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int c = kk * 2 + lk;
      bf16x8 fw[TN], fx[TM];
#pragma unroll
      for (int a = 0; a < TN; ++a) {
        const int r = (wn * TN + a) * 32 + lr;
        fw[a] = as_bf16x8(sWc[r * 8 + (c ^ ((r >> 1) & 7))]);
      }
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const int r = (wm * TM + b) * 32 + lr;
        fx[b] = as_bf16x8(sXc[r * 8 + (c ^ ((r >> 1) & 7))]);
      }
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[a], fx[b], acc[a][b], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds(cur ^ 1);
    __syncthreads();
  }

  // D[i][j]: lane holds j = lane%32 (row of C) and i = 8*(r/4) + 4*(lane/32) + r%4 (column of C).
  // Indices into acc must be compile-time constants or the accumulators leave the register file.
  const bool interior = (m0 + BM <= M) && (n0 + BN <= N) && ((N & 3) == 0);
  static_for<0, TN>([&](auto a) {
    static_for<0, TM>([&](auto b) {
      const int64_t m = m0 + (wm * TM + b) * 32 + lr;
      static_for<0, 4>([&](auto rg) {
        const int64_t n = n0 + (wn * TN + a) * 32 + rg * 8 + lk * 4;
        float v[4] = {acc[a][b][rg * 4 + 0], acc[a][b][rg * 4 + 1], acc[a][b][rg * 4 + 2],
                      acc[a][b][rg * 4 + 3]};
        if (interior) epilogue4_vec<bf16_t, OutT>(v, m, n, N, C, ep);
        else epilogue4_scalar<bf16_t, OutT>(v, m, n, M, N, C, ep);
      });
    });
  });
}

// ------------------------------------------------------------------------------------------------
// fp32: 64x64 tile, K step 16, 256 threads, 4x4 outputs per thread.
template <typename OutT>
__global__ __launch_bounds__(256) void gemm_f32_nt_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                          OutT* __restrict__ C, int64_t M, int64_t N, int64_t K,
                                                          EpiDev ep) {
  __shared__ float sX[16][64 + 4];
  __shared__ float sW[16][64 + 4];
  const int tid = threadIdx.x;
  const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
  const int ty = tid / 16, tx = tid % 16;
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < K; k0 += 16) {
    for (int i = tid; i < 64 * 16; i += 256) {
      const int r = i / 16, c = i % 16;
      sX[c][r] = (m0 + r < M && k0 + c < K) ? X[(m0 + r) * K + k0 + c] : 0.f;
      sW[c][r] = (n0 + r < N && k0 + c < K) ? W[(n0 + r) * K + k0 + c] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sX[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = sW[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) epilogue4_scalar<float, OutT>(acc[i], m0 + ty * 4 + i, n0 + tx * 4, M, N, C, ep);
}

template <typename OutT>
hipError_t launch_generic(const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K, const EpiDev& ep,
                          hipStream_t stream) {
  static bool attr = false;
  return launch_tiles<OutT>(gemm_bf16_nt_generic_kernel<2, 2, 2, 2, OutT>, 128, 128, 256, &attr, X, W, C, M, N, K, ep, 1,
                            stream);
}

template <typename OutT>
hipError_t dispatch_bf16(const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K, const EpiDev& ep,
                         hipStream_t stream) {
  const bool aligned = (((uintptr_t)X | (uintptr_t)W) & 15) == 0;
  int epi = (ep.bias ? E_BIAS : 0) | (ep.gelu ? E_GELU : 0) | (ep.resid ? E_RESID : 0) | (ep.dact_in ? E_DACT : 0) |
            (ep.preact_out ? E_PRE : 0) | (ep.accumulate ? E_ACC : 0);
  if (K % 64 == 0 && aligned && ep.scale == 1.0f) {
    if constexpr (std::is_same<OutT, float>::value) {
      if (epi == 0) return launch_fast<float, 0>(X, W, C, M, N, K, ep, stream);
      if (epi == E_ACC) return launch_fast<float, E_ACC>(X, W, C, M, N, K, ep, stream);
    } else {
      switch (epi) {
        case 0: return launch_fast<bf16_t, 0>(X, W, C, M, N, K, ep, stream);
        case E_BIAS: return launch_fast<bf16_t, E_BIAS>(X, W, C, M, N, K, ep, stream);
        case E_BIAS | E_GELU: return launch_fast<bf16_t, E_BIAS | E_GELU>(X, W, C, M, N, K, ep, stream);
        case E_BIAS | E_RESID: return launch_fast<bf16_t, E_BIAS | E_RESID>(X, W, C, M, N, K, ep, stream);
        case E_BIAS | E_GELU | E_PRE: return launch_fast<bf16_t, E_BIAS | E_GELU | E_PRE>(X, W, C, M, N, K, ep, stream);
        case E_DACT: return launch_fast<bf16_t, E_DACT>(X, W, C, M, N, K, ep, stream);
        default: break;
      }
    }
  }
  return launch_generic<OutT>(X, W, C, M, N, K, ep, stream);
}

}  // namespace

hipError_t gemm_nt(int32_t dtype, const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K,
                   const GemmEpilogue& e, hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
  EpiDev ep{e.bias, e.resid, e.dact_in, e.preact_out, e.gelu, e.accumulate, e.scale};
  const bool out_f32 = e.out_f32 || dtype == PF_DTYPE_F32_;
  if (e.accumulate && !out_f32) return hipErrorInvalidValue;
  if (dtype == PF_DTYPE_BF16_) {
    if (K % 8 != 0) return hipErrorInvalidValue;   // 16-byte operand loads
    if (out_f32) return dispatch_bf16<float>(X, W, C, M, N, K, ep, stream);
    return dispatch_bf16<bf16_t>(X, W, C, M, N, K, ep, stream);
  }
  dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
  hipLaunchKernelGGL(gemm_f32_nt_kernel<float>, grid, dim3(256), 0, stream, (const float*)X, (const float*)W,
                     (float*)C, M, N, K, ep);
  return hipGetLastError();
}

}  // namespace pf
