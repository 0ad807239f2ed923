// Row kernels of the quantised decoder layer around the attention (the decoding pipeline of Section 3.4 in the
// low-precision setting of Section 4.2), and the two offline folds that pipeline rests on.
//
//   k_rmsnorm_quant : x (+ y) -> residual stream, RMSNorm, per-token symmetric int8
//   k_swiglu_quant  : SiLU(gate) * up -> per-token symmetric int8
//   k_fold_qk       : B_Q B_K^T per query head      (set-up, once per model)
//   k_fold_vo       : W_O with B_V folded in        (set-up, once per model)
//
// A decode batch has at most 64 rows, so the row kernels are one workgroup per token: the row is read once, kept in
// registers across the two reductions (sum of squares, largest magnitude) and leaves as packed int8.  They are
// bound by launch latency, not by bandwidth.
#include "wsvd_dev.h"
#include "wsvd_internal.h"

namespace {

constexpr int kRowThreads = 1024;
constexpr int kRowPasses = 4;          // 16 floats per thread: rows of up to 16384 channels

WSVD_DEV float block_sum(float v, float* red) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int k = 0; k < kRowThreads / 64; k++) t += red[k];      // fixed order: the same sum in every thread
  __syncthreads();
  return t;
}
WSVD_DEV float block_max(float v, float* red) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = red[0];
#pragma unroll
  for (int k = 1; k < kRowThreads / 64; k++) t = fmaxf(t, red[k]);
  __syncthreads();
  return t;
}

// int8 codes of 4 values under the activation rule (scale = fp16(max / 127), guarded; round to nearest even; clamp)
WSVD_DEV uint32_t pack_codes(const v4f& f, float sc) {
  uint32_t pk = 0;
#pragma unroll
  for (int e = 0; e < 4; e++) {
    float v = __builtin_rintf(f[e] / sc);
    v = fminf(fmaxf(v, -127.f), 127.f);
    pk |= ((uint32_t)(int)v & 0xFFu) << (8 * e);
  }
  return pk;
}

// x [M, 4 n4] fp32; y (nullable) is added first and the sum written to x_out (the residual stream).
template <bool ADD>
__global__ __launch_bounds__(kRowThreads) void k_rmsnorm_quant(const float* __restrict__ x, const float* __restrict__ y,
                                                               const float* __restrict__ gain, float eps, int n4,
                                                               float* __restrict__ x_out, int8_t* __restrict__ codes,
                                                               uint16_t* __restrict__ scale) {
  __shared__ float red[kRowThreads / 64];
  const int tid = threadIdx.x;
  const size_t row = (size_t)blockIdx.x * n4;
  v4f f[kRowPasses], g[kRowPasses];
#pragma unroll
  for (int it = 0; it < kRowPasses; it++) {
    const int u = min(it * kRowThreads + tid, n4 - 1);           // unconditional, clamped; surplus slots masked below
    f[it] = ((const v4f*)x)[row + u];
    if (ADD) {
      const v4f yy = ((const v4f*)y)[row + u];
      f[it] = f[it] + yy;
    }
    g[it] = ((const v4f*)gain)[u];
  }
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < kRowPasses; it++) {
    const bool on = it * kRowThreads + tid < n4;
    if (ADD && on) ((v4f*)x_out)[row + it * kRowThreads + tid] = f[it];
#pragma unroll
    for (int e = 0; e < 4; e++) ss = on ? fmaf(f[it][e], f[it][e], ss) : ss;
  }
  ss = block_sum(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)(4 * n4) + eps);
  float a = 0.f;
#pragma unroll
  for (int it = 0; it < kRowPasses; it++) {
    const bool on = it * kRowThreads + tid < n4;
#pragma unroll
    for (int e = 0; e < 4; e++) {
      f[it][e] = f[it][e] * inv * g[it][e];
      a = on ? fmaxf(a, fabsf(f[it][e])) : a;
    }
  }
  a = block_max(a, red);
  uint16_t sh = 0x3C00u;
  if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
  const float sc = f16_bits_to_f32(sh);
  uint32_t* dst = (uint32_t*)codes + row;
#pragma unroll
  for (int it = 0; it < kRowPasses; it++) {
    const int u = it * kRowThreads + tid;
    if (u < n4) dst[u] = pack_codes(f[it], sc);
  }
  if (tid == 0) scale[blockIdx.x] = sh;
}

// gu [M, 2F] fp32 (gate in columns [0,F), up in [F,2F)), F = 4 n4.
__global__ __launch_bounds__(kRowThreads) void k_swiglu_quant(const float* __restrict__ gu, int n4,
                                                              int8_t* __restrict__ codes, uint16_t* __restrict__ scale) {
  __shared__ float red[kRowThreads / 64];
  const int tid = threadIdx.x;
  const v4f* grow = (const v4f*)gu + (size_t)blockIdx.x * 2 * n4;
  v4f f[kRowPasses], up[kRowPasses];
#pragma unroll
  for (int it = 0; it < kRowPasses; it++) {
    const int u = min(it * kRowThreads + tid, n4 - 1);
    f[it] = grow[u];
    up[it] = grow[n4 + u];
  }
  float a = 0.f;
#pragma unroll
  for (int it = 0; it < kRowPasses; it++) {
    const bool on = it * kRowThreads + tid < n4;
#pragma unroll
    for (int e = 0; e < 4; e++) {
      const float gt = f[it][e];
      f[it][e] = gt / (1.0f + expf(-gt)) * up[it][e];
      a = on ? fmaxf(a, fabsf(f[it][e])) : a;
    }
  }
  a = block_max(a, red);
  uint16_t sh = 0x3C00u;
  if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
  const float sc = f16_bits_to_f32(sh);
  uint32_t* dst = (uint32_t*)codes + (size_t)blockIdx.x * n4;
#pragma unroll
  for (int it = 0; it < kRowPasses; it++) {
    const int u = it * kRowThreads + tid;
    if (u < n4) dst[u] = pack_codes(f[it], sc);
  }
  if (tid == 0) scale[blockIdx.x] = sh;
}

WSVD_DEV float factor_at(const void* p, size_t i, int dtype) {
  return dtype == WSVD_F32 ? ((const float*)p)[i] : bf16_to_f32(((const uint16_t*)p)[i]);
}

// out[h][i][j] = sum_c B_Q[h][i][c] * B_K[h / G][j][c]; one thread per output
__global__ __launch_bounds__(256) void k_fold_qk(const void* __restrict__ BQ, const void* __restrict__ BK, int dtype, int Hq,
                                                 int G, int rq, int r, int d, float* __restrict__ out) {
  const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (o >= (int64_t)Hq * rq * r) return;
  const int j = (int)(o % r), i = (int)((o / r) % rq), h = (int)(o / ((int64_t)r * rq));
  const size_t qb = ((size_t)h * rq + i) * d, kb = ((size_t)(h / G) * r + j) * d;
  float acc = 0.f;
  for (int c = 0; c < d; c++) acc = fmaf(factor_at(BQ, qb + c, dtype), factor_at(BK, kb + c, dtype), acc);
  out[o] = acc;
}

// out[e][h r + j] = sum_c W_O[e][h d + c] * B_V[h / G][j][c]; one thread per output
__global__ __launch_bounds__(256) void k_fold_vo(const void* __restrict__ BV, int dtype, const float* __restrict__ WO, int E,
                                                 int Hq, int G, int r, int d, float* __restrict__ out) {
  const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (o >= (int64_t)E * Hq * r) return;
  const int j = (int)(o % r), h = (int)((o / r) % Hq);
  const int64_t e = o / ((int64_t)r * Hq);
  const float* w = WO + (size_t)e * Hq * d + (size_t)h * d;
  const size_t vb = ((size_t)(h / G) * r + j) * d;
  float acc = 0.f;
  for (int c = 0; c < d; c++) acc = fmaf(w[c], factor_at(BV, vb + c, dtype), acc);
  out[o] = acc;
}

}  // namespace

hipError_t wsvd_launch_rmsnorm_quant(const float* x, const float* y_add, const float* gain, float eps, int64_t rows,
                                     int64_t cols, float* x_out, int8_t* codes, void* scale_f16, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (cols % 4 != 0 || cols < 4 || cols / 4 > (int64_t)kRowThreads * kRowPasses) return hipErrorInvalidValue;
  if (y_add && !x_out) return hipErrorInvalidValue;
  const int n4 = (int)(cols / 4);
  if (y_add)
    hipLaunchKernelGGL((k_rmsnorm_quant<true>), dim3((unsigned)rows), dim3(kRowThreads), 0, s, x, y_add, gain, eps, n4, x_out,
                       codes, (uint16_t*)scale_f16);
  else
    hipLaunchKernelGGL((k_rmsnorm_quant<false>), dim3((unsigned)rows), dim3(kRowThreads), 0, s, x, y_add, gain, eps, n4, x_out,
                       codes, (uint16_t*)scale_f16);
  return hipGetLastError();
}

hipError_t wsvd_launch_swiglu_quant(const float* gate_up, int64_t rows, int64_t F, int8_t* codes, void* scale_f16, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (F % 4 != 0 || F < 4 || F / 4 > (int64_t)kRowThreads * kRowPasses) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_swiglu_quant, dim3((unsigned)rows), dim3(kRowThreads), 0, s, gate_up, (int)(F / 4), codes,
                     (uint16_t*)scale_f16);
  return hipGetLastError();
}

hipError_t wsvd_launch_fold_qk(const void* BQ, const void* BK, int factor_dtype, int Hq, int Hkv, int rq, int r, int d, float* out,
                               hipStream_t s) {
  const int64_t n = (int64_t)Hq * rq * r;
  hipLaunchKernelGGL(k_fold_qk, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, BQ, BK, factor_dtype, Hq, Hq / Hkv, rq, r, d, out);
  return hipGetLastError();
}

hipError_t wsvd_launch_fold_vo(const void* BV, int factor_dtype, const float* WO, int E, int Hq, int Hkv, int r, int d, float* out,
                               hipStream_t s) {
  const int64_t n = (int64_t)E * Hq * r;
  hipLaunchKernelGGL(k_fold_vo, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, BV, factor_dtype, WO, E, Hq, Hq / Hkv, r, d, out);
  return hipGetLastError();
}
