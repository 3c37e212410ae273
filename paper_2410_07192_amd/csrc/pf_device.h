// Device-side helpers shared by the kernels: bf16 <-> fp32, small vector loads/stores, GELU,
// wavefront reductions.  gfx950 only (wave64).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace pf {

constexpr int32_t PF_DTYPE_F32_ = 0;
constexpr int32_t PF_DTYPE_BF16_ = 1;

struct bf16_t {
  uint16_t bits;
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// two floats to packed bf16 (lo in bits 0..15) with the hardware conversion: round to nearest even
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_bits_to_f32(v.bits); }

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) {
  bf16_t r;
  r.bits = (uint16_t)f32_to_bf16_bits(v);
  return r;
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// 4 consecutive elements (pointer must be aligned to 4 elements)
__device__ __forceinline__ void load4(const float* p, float v[4]) {
  const float4 t = *(const float4*)p;
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load4(const bf16_t* p, float v[4]) {
  const uint2 t = *(const uint2*)p;
  v[0] = bf16_bits_to_f32(t.x & 0xffffu); v[1] = bf16_bits_to_f32(t.x >> 16);
  v[2] = bf16_bits_to_f32(t.y & 0xffffu); v[3] = bf16_bits_to_f32(t.y >> 16);
}
__device__ __forceinline__ void store4(float* p, const float v[4]) {
  *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(bf16_t* p, const float v[4]) {
  uint2 t;
  t.x = pack_bf16x2(v[0], v[1]);
  t.y = pack_bf16x2(v[2], v[3]);
  *(uint2*)p = t;
}

// 8 consecutive elements
__device__ __forceinline__ void load8(const float* p, float v[8]) {
  load4(p, v);
  load4(p + 4, v + 4);
}
__device__ __forceinline__ void load8(const bf16_t* p, float v[8]) {
  const uint4 t = *(const uint4*)p;
  const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = bf16_bits_to_f32(w[i] & 0xffffu);
    v[2 * i + 1] = bf16_bits_to_f32(w[i] >> 16);
  }
}
__device__ __forceinline__ void store8(float* p, const float v[8]) {
  store4(p, v);
  store4(p + 4, v + 4);
}
__device__ __forceinline__ void store8(bf16_t* p, const float v[8]) {
  uint4 t;
  t.x = pack_bf16x2(v[0], v[1]);
  t.y = pack_bf16x2(v[2], v[3]);
  t.z = pack_bf16x2(v[4], v[5]);
  t.w = pack_bf16x2(v[6], v[7]);
  *(uint4*)p = t;
}

// Eight consecutive elements as they come from memory (a first-class vector, so that a load can stay in
// flight until the values are needed), and their conversion to float.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> { typedef uint32_t type __attribute__((ext_vector_type(4))); };
template <> struct Raw8<float> { typedef float type __attribute__((ext_vector_type(8))); };
__device__ __forceinline__ void unpack8(const Raw8<bf16_t>::type& r, float v[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[2 * i] = bf16_bits_to_f32(r[i] & 0xffffu);
    v[2 * i + 1] = bf16_bits_to_f32(r[i] >> 16);
  }
}
__device__ __forceinline__ void unpack8(const Raw8<float>::type& r, float v[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = r[i];
}

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun (absolute error <= 1.5e-7, far
// below the fp32 tolerance of the layer): one exp, one reciprocal and five FMAs instead of the
// library routine, which would otherwise dominate the FFN epilogue.
__device__ __forceinline__ float erf_fast(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));   // 1 ulp reciprocal is ample here
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float y = 1.0f - p * t * __expf(-ax * ax);
  return copysignf(y, x);
}

// GELU in the erf form, x * Phi(x), and its derivative Phi(x) + x * phi(x)
__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erf_fast(x * 0.70710678118654752f)); }
// x * sigmoid(x * (c1 + c3 x^2 + c5 x^4)): minimax fit of the erf form over [-8, 8], absolute error of
// the product <= 2.6e-5 (a hundredth of a bf16 ulp at 1), used where the result is rounded to bf16
// anyway.  One exp2 and one reciprocal; the coefficients carry the factor -log2(e).  x^2 is clamped so the
// polynomial stays positive: beyond |x| = 7 the sigmoid is saturated in fp32 either way.
__device__ __forceinline__ float gelu_bf16_f(float x) {
  const float x2 = fminf(x * x, 49.0f);
  float p = fmaf(1.01426451e-03f, x2, -1.06775722e-01f);   // -log2e * (c5 x2 + c3)
  p = fmaf(p, x2, -2.30112133e+00f);                        // -log2e * c1
  const float e = __builtin_amdgcn_exp2f(x * p);
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}
template <typename T>
__device__ __forceinline__ float gelu_as(float x);   // GELU for results stored as T
template <>
__device__ __forceinline__ float gelu_as<float>(float x) { return gelu_f(x); }
template <>
__device__ __forceinline__ float gelu_as<bf16_t>(float x) { return gelu_bf16_f(x); }

// Phi(x) + x * phi(x) with Phi from the same rational approximation as erf_fast, written out so that the one
// exp(-x^2 / 2) serves both terms: 1 - Phi(|x|) = p(t) * t * exp(-x^2 / 2) / 2 with t = 1 / (1 + 0.3275911 |x| / sqrt 2)
__device__ __forceinline__ float gelu_grad_f(float x) {
  const float ax = fabsf(x);
  const float e = __builtin_amdgcn_exp2f(-0.72134752044448170f * x * x);   // exp(-x^2 / 2)
  const float t = __builtin_amdgcn_rcpf(fmaf(0.23164188843f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float tail = 0.5f * p * t * e;
  return fmaf(x * 0.3989422804014327f, e, x < 0.0f ? tail : 1.0f - tail);
}

// Workgroup ids are dealt round-robin to the 8 XCDs (id % 8).  Returns the work unit of workgroup `pid` such
// that each XCD owns a contiguous range of the n units (its L2 then sees neighbouring units).
__device__ __forceinline__ int64_t xcd_contiguous(int64_t pid, int64_t n) {
  const int64_t q = n >> 3, rem = n & 7;
  const int64_t x = pid & 7, local = pid >> 3;
  return x * q + (x < rem ? x : rem) + local;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}


// One wave-wide copy of 1 KB from global memory straight into LDS (global_load_lds_dwordx4): lane i's 16 bytes at p land
// at LDS byte address dst + 16 i, dst wave-uniform.  The instruction takes the LDS address from M0.  M0 is a register
// the compiler reserves for itself and does not model as clobberable by inline assembly, so the statement puts back
// the value it found: M0 is the same before and after, whatever the compiler keeps there.  Asynchronous: counted by
// vmcnt, not ordered against LDS reads by the compiler (which is why this is not the builtin).
__device__ __forceinline__ void lds_direct_load_1k(uint32_t dst, const void* p) {
  uint32_t saved;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
               : "=&s"(saved)
               : "s"(dst), "v"(p)
               : "memory");
}

}  // namespace pf
