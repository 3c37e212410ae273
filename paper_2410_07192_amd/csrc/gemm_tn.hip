// Weight-gradient GEMM for bf16 training:  C[M][N] (fp32) += A^T B  with A [K][M] and B [K][N] row-major,
// i.e. both operands as the layer left them in memory (tokens are the slow index): dW = dY^T X needs no
// transposed copies.  Optionally colsum[m] += sum over k of A[k][m], which is the bias gradient of the same layer.
//
// 128x128 tiles, 4 waves (2x2, wave tile 64x64 = 2x2 MFMA 32x32x16 tiles), K steps of 64, two LDS stages
// of 32 KB, two workgroups per CU.  Operand slabs go global -> LDS directly, 4 k-rows x 256 bytes per wave
// instruction, in the [k][m] order they have in memory.  MFMA wants, per lane, eight consecutive k of one m:
// ds_read_b64_tr_b16 delivers exactly that from a k-major image (a 16-lane group reads a 4 k x 16 m block and
// every lane receives the four k of its own m), two reads per fragment.  The 16-byte chunks of a k-row are
// XOR-swizzled by 4 * (k % 4) (on the global side of the copy) so that the four rows a half-wave reads fall
// on disjoint banks.
// Split K: gridDim.y workgroups share a tile, each over K / gridDim.y; the fp32 tile goes through LDS and is
// added to C with fp32 atomics in coalesced order (plain read-add-write when K is not split).  The column sum
// comes from one more MFMA per A fragment against a fragment of ones, on the waves of the first tile column.
#include <type_traits>

#include "pf_device.h"
#include "pf_kernels.h"

namespace pf {
namespace {

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(3))) char* lds_char_ptr;

template <int I, int N, class F>
__device__ __forceinline__ void unrolled(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    unrolled<I + 1, N>(f);
  }
}

template <bool COLSUM>
__global__ __launch_bounds__(256, 2) void gemm_bf16_tn_acc_kernel(const bf16_t* __restrict__ A,
                                                                  const bf16_t* __restrict__ B, float* __restrict__ C,
                                                                  float* __restrict__ colsum, int64_t M, int64_t N,
                                                                  int64_t K, int32_t tiles_m, int32_t tiles_n) {
  constexpr int BM = 128, BN = 128, TM = 2, TN = 2, NW = 4, STAGE = 32768, BOFF = 16384;
  extern __shared__ char smem[];
  const int64_t tile = xcd_contiguous(blockIdx.x, (int64_t)tiles_m * tiles_n);
  const int32_t tn_i = (int32_t)(tile % tiles_n), tm_i = (int32_t)(tile / tiles_n);
  const int64_t m0 = (int64_t)tm_i * BM, n0 = (int64_t)tn_i * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int lr = lane & 31, lk = lane >> 5;
  const int64_t k_len = K / gridDim.y;
  const int64_t kbeg = (int64_t)blockIdx.y * k_len;
  const int64_t nk = k_len / 64;

  // global source of this lane for each of the 8 copies the wave issues per stage (4 of A, 4 of B): copy q
  // covers k-rows 4q..4q+3 of the step; the lane takes chunk (lane % 16) ^ 4 * (lane / 16) of row lane / 16
  const int krow = lane >> 4;
  const int cglob = (lane & 15) ^ (4 * krow);
  const bf16_t* src[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int q = wave + 4 * i;   // 0..15 A, 16..31 B
    const bool isa = q < 16;
    const int64_t ld = isa ? M : N;
    int64_t col = (isa ? m0 : n0) + cglob * 8;
    if (col + 8 > ld) col = ld - 8;   // tile edge: any valid chunk, the result is discarded
    src[i] = (isa ? A : B) + (kbeg + (q & 15) * 4 + krow) * ld + col;
  }
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_ptr)smem);
  auto issue = [&](auto ic, int stage, int64_t kstep) {
    constexpr int i = decltype(ic)::value;
    const int q = wave + 4 * i;
    const uint32_t dst =
        __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)(stage * STAGE + (q < 16 ? 0 : BOFF) + (q & 15) * 1024));
    const bf16_t* p = src[i] + kstep * 64 * (q < 16 ? M : N);
    lds_direct_load_1k(dst, p);
  };

  // fragment addressing: lane 16 g + i points at k-row (g / 2) * 8 + r * 4 + i / 4 of the 16-row substep and at
  // the four columns from (g % 2) * 16 + 4 * (i % 4) of its 32-column block, and receives column
  // (g % 2) * 16 + i with the four k of read r: MFMA row lane % 32, k half lane / 32
  const int g = lane >> 4, li = lane & 15, kq = li >> 2;
  int offA[TM], offB[TN];
#pragma unroll
  for (int b = 0; b < TM; ++b) {
    const int colb = ((wm * TM + b) * 32 + (g & 1) * 16 + 4 * (li & 3)) * 2;
    offA[b] = ((g >> 1) * 8 + kq) * 256 + (((colb >> 4) ^ (4 * kq)) << 4) + (colb & 15);
  }
#pragma unroll
  for (int a = 0; a < TN; ++a) {
    const int colb = ((wn * TN + a) * 32 + (g & 1) * 16 + 4 * (li & 3)) * 2;
    offB[a] = BOFF + ((g >> 1) * 8 + kq) * 256 + (((colb >> 4) ^ (4 * kq)) << 4) + (colb & 15);
  }
  auto frag = [&](int stage, int off, int ks) {
    lds_char_ptr base = (lds_char_ptr)(lds_void_ptr)smem + stage * STAGE + off + ks * 16 * 256;
    const v4s r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)base);
    const v4s r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(base + 4 * 256));
    v8s o;
    o[0] = r0[0]; o[1] = r0[1]; o[2] = r0[2]; o[3] = r0[3];
    o[4] = r1[0]; o[5] = r1[1]; o[6] = r1[2]; o[7] = r1[3];
    return __builtin_bit_cast(bf16x8, o);
  };

  f32x16 acc[TN][TM], csum[TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
#pragma unroll
  for (int b = 0; b < TM; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) csum[b][r] = 0.f;
  v8s ones_s;
#pragma unroll
  for (int j = 0; j < 8; ++j) ones_s[j] = (short)0x3f80;   // bf16 1.0
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_s);
  const bool do_sum = COLSUM && tn_i == 0 && wn == 0;

  unrolled<0, 8>([&](auto i) { issue(i, 0, 0); });
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int cur = (int)(kt & 1);
    // the other stage was last read before the barrier that ended the previous step
    if (kt + 1 < nk) unrolled<0, 8>([&](auto i) { issue(i, cur ^ 1, kt + 1); });
    // fragments of substep ks + 1 are requested before the MFMAs of substep ks are issued
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int b = 0; b < TM; ++b) fa[0][b] = frag(cur, offA[b], 0);
#pragma unroll
    for (int a = 0; a < TN; ++a) fb[0][a] = frag(cur, offB[a], 0);
    unrolled<0, 4>([&](auto ksc) {
      constexpr int ks = decltype(ksc)::value, buf = ks & 1;
      if constexpr (ks + 1 < 4) {
#pragma unroll
        for (int b = 0; b < TM; ++b) fa[buf ^ 1][b] = frag(cur, offA[b], ks + 1);
#pragma unroll
        for (int a = 0; a < TN; ++a) fb[buf ^ 1][a] = frag(cur, offB[a], ks + 1);
      }
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][a], fa[buf][b], acc[a][b], 0, 0, 0);
      if constexpr (COLSUM) {
        if (do_sum) {
#pragma unroll
          for (int b = 0; b < TM; ++b)
            csum[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, fa[buf][b], csum[b], 0, 0, 0);
        }
      }
    });
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
  }

  // D[i][j]: lane holds j = lane % 32 (row of C) and i = 8 * (r / 4) + 4 * (lane / 32) + r % 4 (column of C).
  if constexpr (COLSUM) {
    // every row i of ones x A equals the column sums: row 0 sits in register 0 of lanes 0..31
    if (do_sum && lane < 32) {
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const int64_t m = m0 + (wm * TM + b) * 32 + lane;
        if (m < M) unsafeAtomicAdd(colsum + m, csum[b][0]);
      }
    }
  }
  // the fp32 tile takes both LDS stages (row-major, 16-byte units XOR-swizzled by row) and leaves in rows
  float* stf = (float*)smem;
  constexpr int UNITS = BN / 4, NT = 64 * NW;
  unrolled<0, TN>([&](auto a) {
    unrolled<0, TM>([&](auto b) {
      const int row = (wm * TM + b) * 32 + lr;
      unrolled<0, 4>([&](auto rg) {
        const int unit = ((wn * TN + a) * 32 + rg * 8 + lk * 4) / 4;
        *(float4*)(stf + row * BN + ((unit ^ (row & (UNITS - 1))) * 4)) =
            make_float4(acc[a][b][rg * 4 + 0], acc[a][b][rg * 4 + 1], acc[a][b][rg * 4 + 2], acc[a][b][rg * 4 + 3]);
      });
    });
  });
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __builtin_amdgcn_s_barrier();
  const bool split = gridDim.y > 1;
#pragma unroll 8
  for (int i = 0; i < BM * BN / NT; ++i) {
    const int e = i * NT + tid, row = e / BN, col = e % BN;
    const float v = stf[row * BN + (((col >> 2) ^ (row & (UNITS - 1))) * 4) + (col & 3)];
    if (m0 + row < M && n0 + col < N) {
      float* p = C + (m0 + row) * N + n0 + col;
      if (split) unsafeAtomicAdd(p, v);
      else *p += v;
    }
  }
}

}  // namespace

bool gemm_tn_acc_supported(int32_t dtype, const void* A, const void* B, int64_t M, int64_t N, int64_t K) {
  return dtype == PF_DTYPE_BF16_ && M >= 8 && N >= 8 && M % 8 == 0 && N % 8 == 0 && K >= 64 && K % 64 == 0 &&
         (((uintptr_t)A | (uintptr_t)B) & 15) == 0;
}

// The 128x128 tiles of this kernel reach about 650 TFLOP/s; the NT kernel's 256-wide tiles about 900 on results
// large enough to fill the chip with them, but it needs both operands transposed first (4 K (M + N) bytes at about
// 4 TB/s).  Equating the two gives M N / (M + N) = 1170: below that, or when 256x256 tiles would leave CUs idle,
// this kernel is the faster way to a weight gradient.
bool gemm_tn_acc_preferred(int64_t M, int64_t N, int64_t K) {
  (void)K;   // both sides of the comparison are proportional to K
  const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
  return big_tiles < 256 || M * N < 1170 * (M + N);
}

hipError_t gemm_tn_acc(int32_t dtype, const void* A, const void* B, float* C, float* colsum, int64_t M, int64_t N,
                       int64_t K, hipStream_t stream) {
  if (!gemm_tn_acc_supported(dtype, A, B, M, N, K)) return hipErrorInvalidValue;
  const int64_t tiles_m = (M + 127) / 128, tiles_n = (N + 127) / 128, tiles = tiles_m * tiles_n;
  if (tiles > 0x7fffffff) return hipErrorInvalidValue;
  // Slices of K per tile.  Measured on MI355X: a K step takes 0.93 us on a workgroup that has its CU to itself and
  // 1.22 us on a pair that shares one; the atomic adds of a slice cost 0.67 us per MiB of fp32 tile.  Two
  // workgroups per CU are resident; a slice keeps at least 8 steps.
  int best = 1;
  double best_t = -1.0;
  for (int s = 1; s <= 16; s *= 2) {
    if (s > 1 && (K % (64 * s) != 0 || K / (64 * s) < 8 || tiles * s > 512)) break;
    const int64_t wgs = tiles * s, rounds = (wgs + 511) / 512;
    const double steps = (double)(K / (64 * s)) + 4.0;
    double t = (double)rounds * steps * (wgs <= 256 ? 0.93 : 1.22);
    if (s > 1) t += (double)M * (double)N * 4.0 * s / 1048576.0 * 0.67;
    if (best_t < 0 || t < best_t) {
      best_t = t;
      best = s;
    }
  }
  static bool attr[2] = {false, false};
  auto launch = [&](auto kern, bool* attr_set) {
    if (!*attr_set) {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
      if (e != hipSuccess) return e;
      *attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles, (unsigned)best), dim3(256), 65536, stream, (const bf16_t*)A,
                       (const bf16_t*)B, C, colsum, M, N, K, (int32_t)tiles_m, (int32_t)tiles_n);
    return hipGetLastError();
  };
  if (colsum) return launch(gemm_bf16_tn_acc_kernel<true>, &attr[0]);
  return launch(gemm_bf16_tn_acc_kernel<false>, &attr[1]);
}

}  // namespace pf
