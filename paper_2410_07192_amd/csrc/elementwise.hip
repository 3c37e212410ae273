// HBM-bound kernels: LayerNorm forward and embedding gather.  One wavefront owns one row; each lane
// moves 8 consecutive elements per access (16 bytes of bf16, 32 of fp32) so a wave touches whole
// cache lines; the row stays in registers between the statistics pass and the normalisation, so
// every element is read once and written once.
#include "pf_kernels.h"
#include "pf_device.h"

namespace pf {
namespace {

template <typename T, int ITER>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                            const T* __restrict__ b, T* __restrict__ y,
                                                            float* __restrict__ mean_out,
                                                            float* __restrict__ rstd_out, int64_t rows, int32_t d,
                                                            float eps, const uint4* __restrict__ warm, int64_t warm_n) {
  // Optional side job: read warm_n 16-byte pieces (the weights of the GEMMs that follow) and drop them, so that
  // they sit in the memory-side cache when a GEMM's first round of tiles asks for them all at once.  A layer's
  // weights were last used a whole pass over the model earlier and are long evicted; with cold weights the
  // QKV and FFN GEMMs of the 12-layer encoder workload take 3-7 us longer each (measured on one machine, in the
  // same process, with and without), against 1.6 us that the extra reads add to this kernel.
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < warm_n; i += (int64_t)gridDim.x * 256) {
    const uint4 v = warm[i];
    asm volatile("" ::"v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w));
  }
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  // every load of the wave is issued up front and stays raw until it is needed (x first, then gain and bias,
  // which the statistics leave time to arrive); a group of 8 columns past the end reads column 0 and is not used
  typedef typename Raw8<T>::type raw_t;
  const T* xr = x + row * d;
  raw_t xraw[ITER], graw[ITER], braw[ITER];
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int c = (i * 64 + lane) * 8;
    xraw[i] = *(const raw_t*)(xr + (c < d ? c : 0));
  }
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int c = (i * 64 + lane) * 8;
    graw[i] = *(const raw_t*)(g + (c < d ? c : 0));
    braw[i] = *(const raw_t*)(b + (c < d ? c : 0));
  }
  __builtin_amdgcn_sched_barrier(0);   // nothing that waits for the first load moves above the last one
  float v[ITER][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int c = (i * 64 + lane) * 8;
    unpack8(xraw[i], v[i]);
    if (c < d) {
#pragma unroll
      for (int j = 0; j < 8; ++j) s += v[i][j];
    }
  }
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (c < d) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float t = v[i][j] - mean;
        q += t * t;
      }
    }
  }
  const float rstd = rsqrtf(wave_sum(q) / (float)d + eps);
  if (lane == 0) {
    if (mean_out) mean_out[row] = mean;
    if (rstd_out) rstd_out[row] = rstd;
  }
  T* yr = y + row * d;
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int c = (i * 64 + lane) * 8;
    float gg[8], bb[8], o[8];
    unpack8(graw[i], gg);
    unpack8(braw[i], bb);
    if (c < d) {
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = (v[i][j] - mean) * rstd * gg[j] + bb[j];
      store8(yr + c, o);
    }
  }
}

template <typename T>
hipError_t launch_ln(const void* x, const void* g, const void* b, void* y, float* mo, float* ro, int64_t rows,
                     int32_t d, float eps, const uint4* warm, int64_t warm_n, hipStream_t st) {
  const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  const int iters = (d + 511) / 512;
#define PF_LN(I)                                                                                             \
  hipLaunchKernelGGL((layernorm_fwd_kernel<T, I>), grid, block, 0, st, (const T*)x, (const T*)g, (const T*)b, \
                     (T*)y, mo, ro, rows, d, eps, warm, warm_n)
  if (iters <= 1) PF_LN(1);
  else if (iters <= 2) PF_LN(2);
  else if (iters <= 4) PF_LN(4);
  else if (iters <= 8) PF_LN(8);
  else if (iters <= 16) PF_LN(16);
  else return hipErrorInvalidValue;
#undef PF_LN
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const int32_t* __restrict__ ids, const T* __restrict__ tok,
                                                        const T* __restrict__ pos, T* __restrict__ x, int64_t tokens,
                                                        int32_t S, int32_t d, int32_t V) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= tokens) return;
  const int32_t id = ids[t];
  const bool ok = id >= 0 && id < V;
  const T* tr = tok + (int64_t)(ok ? id : 0) * d;
  const T* pr = pos + (t % S) * d;
  T* xr = x + t * d;
  for (int c = lane * 8; c < d; c += 512) {
    float a[8], p[8];
    load8(pr + c, p);
    if (ok) {
      load8(tr + c, a);
#pragma unroll
      for (int j = 0; j < 8; ++j) p[j] += a[j];
    }
    store8(xr + c, p);
  }
}

}  // namespace

hipError_t layernorm_fwd(int32_t dtype, const void* x, const void* g, const void* b, void* y, float* mean_out,
                         float* rstd_out, int64_t rows, int32_t d, float eps, hipStream_t stream, const void* warm,
                         int64_t warm_bytes) {
  if (rows <= 0 || d <= 0 || d % 8 != 0 || d > 8192) return hipErrorInvalidValue;
  // whole 16-byte pieces inside [warm, warm + warm_bytes)
  const uintptr_t w0 = ((uintptr_t)warm + 15) & ~(uintptr_t)15;
  const int64_t skip = (int64_t)(w0 - (uintptr_t)warm);
  const int64_t warm_n = (warm && warm_bytes > skip) ? (warm_bytes - skip) / 16 : 0;
  if (dtype == PF_DTYPE_BF16_)
    return launch_ln<bf16_t>(x, g, b, y, mean_out, rstd_out, rows, d, eps, (const uint4*)w0, warm_n, stream);
  return launch_ln<float>(x, g, b, y, mean_out, rstd_out, rows, d, eps, (const uint4*)w0, warm_n, stream);
}

hipError_t embed_fwd(int32_t dtype, const int32_t* ids, const void* tok, const void* pos, void* x, int64_t tokens,
                     int32_t S, int32_t d, int32_t V, hipStream_t stream) {
  if (tokens <= 0 || d <= 0 || d % 8 != 0 || S <= 0 || V <= 0) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((tokens + 3) / 4)), block(256);
  if (dtype == PF_DTYPE_BF16_)
    hipLaunchKernelGGL(embed_fwd_kernel<bf16_t>, grid, block, 0, stream, ids, (const bf16_t*)tok,
                       (const bf16_t*)pos, (bf16_t*)x, tokens, S, d, V);
  else
    hipLaunchKernelGGL(embed_fwd_kernel<float>, grid, block, 0, stream, ids, (const float*)tok, (const float*)pos,
                       (float*)x, tokens, S, d, V);
  return hipGetLastError();
}

}  // namespace pf
