// GEMM kernels for gfx950:  C[M,N] = epilogue( X[M,K] * W[N,K]^T ).
//
// bf16 path: 32x32x16 bf16 MFMA, fp32 accumulators.  A workgroup of WGM x WGN waves owns a
// (WGM*TM*32) x (WGN*TN*32) tile of C and walks K in steps of 64.  Both operand tiles are staged in
// LDS as 16-byte chunks (8 bf16 along K) with an XOR swizzle so that the 32 rows a wave reads for one
// MFMA operand fall into distinct banks; LDS is double buffered and the next K step's global loads
// are issued before the MFMAs of the current one.  The weight tile is the MFMA "A" operand and the
// activation tile the "B" operand, so that each lane ends up with 4 consecutive output columns of
// one output row: bias / residual / GELU are applied in registers and stored as 8-byte pieces.
// Workgroup ids are remapped so that each of the 8 XCDs (ids are dealt round-robin to them) works on
// a contiguous range of tiles and its L2 sees each operand panel once.
//
// fp32 path (small parity workload only): plain LDS-tiled FMA kernel with the same epilogue.
#include "pf_kernels.h"
#include "pf_device.h"

namespace pf {
namespace {

struct EpiDev {
  const void* bias;
  const void* resid;
  const void* dact_in;
  void* preact_out;
  int32_t gelu, accumulate;
  float scale;
};

// Epilogue for 4 consecutive columns n0..n0+3 of row m.  T = storage type of bias / resid / aux,
// OutT = type of C.
template <typename T, typename OutT>
__device__ __forceinline__ void epilogue4(float v[4], int64_t m, int64_t n0, int64_t M, int64_t N, OutT* C,
                                          const EpiDev& ep) {
  if (m >= M || n0 >= N) return;
  const int64_t off = m * N + n0;
  const bool full = (n0 + 3 < N) && ((N & 3) == 0);
  const T* bias = (const T*)ep.bias;
  const T* resid = (const T*)ep.resid;
  const T* dact = (const T*)ep.dact_in;
  T* pre = (T*)ep.preact_out;
  if (full) {
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
      for (int j = 0; j < 4; ++j) v[j] = gelu_f(v[j]);
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
  } else {
    for (int j = 0; j < 4 && n0 + j < N; ++j) {
      float x = v[j] * ep.scale;
      if (bias) x += to_f32(bias[n0 + j]);
      if (pre) pre[off + j] = from_f32<T>(x);
      if (ep.gelu) x = gelu_f(x);
      if (dact) x *= gelu_grad_f(to_f32(dact[off + j]));
      if (resid) x += to_f32(resid[off + j]);
      if (ep.accumulate) x += to_f32(C[off + j]);
      C[off + j] = from_f32<OutT>(x);
    }
  }
}

// workgroup id -> tile id such that XCD x (ids congruent x mod 8) gets a contiguous tile range
__device__ __forceinline__ int64_t xcd_tile(int64_t pid, int64_t n_tiles) {
  const int64_t q = n_tiles >> 3, rem = n_tiles & 7;
  const int64_t x = pid & 7, local = pid >> 3;
  return x * q + (x < rem ? x : rem) + local;
}

// ------------------------------------------------------------------------------------------------
template <int WGM, int WGN, int TM, int TN, typename OutT>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_nt_kernel(
    const bf16_t* __restrict__ X, const bf16_t* __restrict__ W, OutT* __restrict__ C, int64_t M, int64_t N,
    int64_t K, EpiDev ep, int32_t tiles_m, int32_t tiles_n, int32_t group_m) {
  constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32, NT = 64 * WGM * WGN;
  constexpr int XCH = BM * 8 / NT, WCH = BN * 8 / NT;   // 16-byte chunks per thread per K step
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile / thread mismatch");
  extern __shared__ uint4 smem[];
  // buffer b: X tile at smem + b*(BM+BN)*8, W tile right after it

  // tile coordinates: contiguous range per XCD, grouped so `group_m` row tiles share the sweep over N
  const int64_t tile = xcd_tile(blockIdx.x, (int64_t)tiles_m * tiles_n);
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

  // D[i][j]: lane holds j = lane%32 (row of C) and i = 8*(r/4) + 4*(lane/32) + r%4 (column of C)
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      const int64_t m = m0 + (wm * TM + b) * 32 + lr;
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int64_t n = n0 + (wn * TN + a) * 32 + rg * 8 + lk * 4;
        float v[4] = {acc[a][b][rg * 4 + 0], acc[a][b][rg * 4 + 1], acc[a][b][rg * 4 + 2],
                      acc[a][b][rg * 4 + 3]};
        epilogue4<bf16_t, OutT>(v, m, n, M, N, C, ep);
      }
    }
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
  for (int i = 0; i < 4; ++i) epilogue4<float, OutT>(acc[i], m0 + ty * 4 + i, n0 + tx * 4, M, N, C, ep);
}

template <int WGM, int WGN, int TM, int TN, typename OutT>
hipError_t launch_bf16(const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K, const EpiDev& ep,
                       hipStream_t stream) {
  constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
  const int64_t tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const size_t lds = (size_t)2 * (BM + BN) * 8 * sizeof(uint4);
  auto kern = gemm_bf16_nt_kernel<WGM, WGN, TM, TN, OutT>;
  static bool attr_set = false;   // raise the dynamic-LDS limit once per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int32_t group_m = 8;
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WGM * WGN), lds, stream,
                     (const bf16_t*)X, (const bf16_t*)W, (OutT*)C, M, N, K, ep, (int32_t)tiles_m, (int32_t)tiles_n,
                     group_m);
  return hipGetLastError();
}

template <typename OutT>
hipError_t dispatch_bf16(const void* X, const void* W, void* C, int64_t M, int64_t N, int64_t K, const EpiDev& ep,
                         hipStream_t stream) {
  // Pick the largest tile that still gives every CU (256 of them) at least ~2 tiles of work.
  const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
  const int64_t t128x256 = ((M + 127) / 128) * ((N + 255) / 256);
  if (t256 >= 512) return launch_bf16<2, 2, 4, 4, OutT>(X, W, C, M, N, K, ep, stream);
  if (t128x256 >= 384) return launch_bf16<2, 2, 2, 4, OutT>(X, W, C, M, N, K, ep, stream);
  return launch_bf16<2, 2, 2, 2, OutT>(X, W, C, M, N, K, ep, stream);
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
