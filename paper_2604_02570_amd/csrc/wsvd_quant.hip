// Quantiser entry points and the logical <-> device cache layout copies.
#include "wsvd_dev.h"
#include "wsvd_internal.h"

// ---------------------------------------------------------------- wsvd_quantize_rows
// One thread per latent row: the row sits in registers and goes through the same quantize_row_*
// routine the append kernel uses, so both produce identical bits on identical fp32 inputs.
template <int R>
__global__ __launch_bounds__(256) void k_quantize_rows_i8(const float* __restrict__ c, int64_t n_rows,
                                                           int8_t* __restrict__ codes, uint16_t* __restrict__ scale) {
  int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_rows) return;
  float v[R];
  const v4f* src = (const v4f*)(c + row * R);
#pragma unroll
  for (int i = 0; i < R / 4; i++) { v4f t = src[i]; v[4 * i] = t[0]; v[4 * i + 1] = t[1]; v[4 * i + 2] = t[2]; v[4 * i + 3] = t[3]; }
  int8_t q[R];
  uint16_t sh = quantize_row_i8<R>(v, q);
  int* dst = (int*)(codes + row * R);
#pragma unroll
  for (int i = 0; i < R / 4; i++)
    dst[i] = (int)((uint32_t)(uint8_t)q[4 * i] | ((uint32_t)(uint8_t)q[4 * i + 1] << 8) | ((uint32_t)(uint8_t)q[4 * i + 2] << 16) |
                   ((uint32_t)(uint8_t)q[4 * i + 3] << 24));
  scale[row] = sh;
}

template <int R>
__global__ __launch_bounds__(256) void k_quantize_rows_i4(const float* __restrict__ c, int64_t n_rows,
                                                           uint8_t* __restrict__ codes, uint16_t* __restrict__ meta) {
  int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_rows) return;
  float v[R];
  const v4f* src = (const v4f*)(c + row * R);
#pragma unroll
  for (int i = 0; i < R / 4; i++) { v4f t = src[i]; v[4 * i] = t[0]; v[4 * i + 1] = t[1]; v[4 * i + 2] = t[2]; v[4 * i + 3] = t[3]; }
  uint8_t q[R];
  uint16_t sh, zh;
  quantize_row_i4<R>(v, q, &sh, &zh);
  int* dst = (int*)(codes + row * (R / 2));
#pragma unroll
  for (int i = 0; i < R / 8; i++) {
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 8; k++) w |= (uint32_t)q[8 * i + k] << (4 * k);   // element 2i low nibble, 2i+1 high nibble
    dst[i] = (int)w;
  }
  meta[2 * row] = sh;
  meta[2 * row + 1] = zh;
}

hipError_t wsvd_launch_quantize_rows(int latent_dtype, int rank, const float* c, int64_t n_rows, void* codes, void* meta,
                                     hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  dim3 grid((unsigned)((n_rows + 255) / 256)), block(256);
  if (latent_dtype == WSVD_I8) {
    if (rank == 32) hipLaunchKernelGGL(k_quantize_rows_i8<32>, grid, block, 0, s, c, n_rows, (int8_t*)codes, (uint16_t*)meta);
    else if (rank == 64) hipLaunchKernelGGL(k_quantize_rows_i8<64>, grid, block, 0, s, c, n_rows, (int8_t*)codes, (uint16_t*)meta);
    else if (rank == 96) hipLaunchKernelGGL(k_quantize_rows_i8<96>, grid, block, 0, s, c, n_rows, (int8_t*)codes, (uint16_t*)meta);
    else if (rank == 128) hipLaunchKernelGGL(k_quantize_rows_i8<128>, grid, block, 0, s, c, n_rows, (int8_t*)codes, (uint16_t*)meta);
    else return hipErrorInvalidValue;
  } else if (latent_dtype == WSVD_I4 && rank == 32) {
    hipLaunchKernelGGL(k_quantize_rows_i4<32>, grid, block, 0, s, c, n_rows, (uint8_t*)codes, (uint16_t*)meta);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------- per-token activation quantiser
// One workgroup per row: abs-max over the row (wave DPP + LDS), then the I8 rule element-wise.
__global__ __launch_bounds__(256) void k_quantize_act_i8(const void* __restrict__ x, int x_dtype, int64_t cols,
                                                          int8_t* __restrict__ codes, uint16_t* __restrict__ scale) {
  __shared__ float red[4];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  float a = 0.f;
  for (int64_t cidx = tid; cidx < cols; cidx += 256) a = fmaxf(a, fabsf(load_as_f32(x, row * cols + cidx, x_dtype)));
  a = wave_max(a);
  if ((tid & 63) == 0) red[tid >> 6] = a;
  __syncthreads();
  a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  uint16_t sh = 0x3C00u;
  if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
  const float sc = f16_bits_to_f32(sh);
  for (int64_t cidx = tid; cidx < cols; cidx += 256) {
    float v = __builtin_rintf(load_as_f32(x, row * cols + cidx, x_dtype) / sc);
    v = fminf(fmaxf(v, -127.f), 127.f);
    codes[row * cols + cidx] = (int8_t)(int)v;
  }
  if (tid == 0) scale[row] = sh;
}

// Rows of up to 16384 elements: the row is read ONCE, 16 bytes per thread and pass with every pass in flight
// together, kept in registers across the abs-max reduction, and the codes leave as packed dwords.  Same arithmetic
// per element as the kernel above (max is exact in any order), so the stored bits are identical.
constexpr int kActThreads = 1024;
constexpr int kActPasses = 4;
template <int ESZ>   // 4: fp32, 2: bf16
__global__ __launch_bounds__(kActThreads) void k_quantize_act_i8_row(const void* __restrict__ x, int n16 /* 16-byte units per row */,
                                                                      int8_t* __restrict__ codes, uint16_t* __restrict__ scale) {
  constexpr int EPU = 16 / ESZ;      // elements per 16-byte unit
  __shared__ float red[kActThreads / 64];
  const int tid = threadIdx.x;
  const v4i* src = (const v4i*)x + (size_t)blockIdx.x * n16;
  v4i raw[kActPasses];
#pragma unroll
  for (int it = 0; it < kActPasses; it++) raw[it] = src[min(it * kActThreads + tid, n16 - 1)];   // unconditional, clamped
  float f[kActPasses][EPU];
  float a = 0.f;
#pragma unroll
  for (int it = 0; it < kActPasses; it++)
#pragma unroll
    for (int e = 0; e < EPU; e++) {
      if (ESZ == 4) f[it][e] = __int_as_float(raw[it][e]);
      else f[it][e] = __uint_as_float((e & 1) ? ((uint32_t)raw[it][e >> 1] & 0xFFFF0000u) : ((uint32_t)raw[it][e >> 1] << 16));
      a = fmaxf(a, fabsf(f[it][e]));     // clamped duplicates repeat an element of the row: harmless for a max
    }
  a = wave_max(a);
  if ((tid & 63) == 0) red[tid >> 6] = a;
  __syncthreads();
  a = red[0];
#pragma unroll
  for (int k = 1; k < kActThreads / 64; k++) a = fmaxf(a, red[k]);
  uint16_t sh = 0x3C00u;
  if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
  const float sc = f16_bits_to_f32(sh);
  uint32_t* dst = (uint32_t*)(codes + (size_t)blockIdx.x * n16 * EPU);
#pragma unroll
  for (int it = 0; it < kActPasses; it++) {
    const int u = it * kActThreads + tid;
    if (u < n16) {
#pragma unroll
      for (int w4 = 0; w4 < EPU / 4; w4++) {
        uint32_t pk = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
          float v = __builtin_rintf(f[it][w4 * 4 + e] / sc);
          v = fminf(fmaxf(v, -127.f), 127.f);
          pk |= ((uint32_t)(int)v & 0xFFu) << (8 * e);
        }
        dst[(size_t)u * (EPU / 4) + w4] = pk;
      }
    }
  }
  if (tid == 0) scale[blockIdx.x] = sh;
}

hipError_t wsvd_launch_quantize_act_i8(const void* x, int x_dtype, int64_t rows, int64_t cols, int8_t* codes,
                                       void* scale_f16, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  const int esz = x_dtype == WSVD_F32 ? 4 : 2;
  const int epu = 16 / esz;
  const bool fast = (x_dtype == WSVD_F32 || x_dtype == WSVD_BF16) && cols % epu == 0 &&
                    cols / epu <= (int64_t)kActThreads * kActPasses && ((uintptr_t)x & 15u) == 0 && ((uintptr_t)codes & 3u) == 0;
  if (fast) {
    const int n16 = (int)(cols / epu);
    if (esz == 4) hipLaunchKernelGGL((k_quantize_act_i8_row<4>), dim3((unsigned)rows), dim3(kActThreads), 0, s, x, n16, codes, (uint16_t*)scale_f16);
    else hipLaunchKernelGGL((k_quantize_act_i8_row<2>), dim3((unsigned)rows), dim3(kActThreads), 0, s, x, n16, codes, (uint16_t*)scale_f16);
  } else {
    hipLaunchKernelGGL(k_quantize_act_i8, dim3((unsigned)rows), dim3(256), 0, s, x, x_dtype, cols, codes, (uint16_t*)scale_f16);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------- logical <-> device layout copies
struct CopyArgs {
  uint8_t* lcodes;   // logical [B*Hkv, n_rows, row_bytes]
  uint16_t* lmeta;   // logical [B*Hkv, n_rows(,2)]
  uint8_t* dcodes;   // device plane
  uint16_t* dmeta;
  int n_planes;      // B*Hkv
  int t_cap, t0, n_rows, rank, dtype, plane;
  int to_device;
};

// F32 / BF16 / I8 and the I4 K plane: one thread per logical byte (each maps to exactly one device byte).
__global__ __launch_bounds__(256) void k_cache_copy_bytes(CopyArgs a) {
  const int rb = row_code_bytes(a.rank, a.dtype);
  const int64_t total = (int64_t)a.n_planes * a.n_rows * rb;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int byte = (int)(i % rb);
  const int64_t rowi = i / rb;
  const int tr = (int)(rowi % a.n_rows);
  const int64_t ph = rowi / a.n_rows;
  const int t = a.t0 + tr;
  size_t plane_bytes = (size_t)a.t_cap * rb;
  size_t off;
  if (a.dtype == WSVD_I8) {
    off = a.plane == 0 ? i8_k_offset(t, byte, a.rank) : i8_v_offset(t, byte, a.rank);
  } else if (a.dtype == WSVD_I4) {
    int nib;
    off = i4_k_offset(t, 2 * byte, &nib);     // K plane only: dims (2*byte, 2*byte+1) share a device byte too
  } else {
    off = (size_t)t * rb + byte;
  }
  uint8_t* dp = a.dcodes + ph * plane_bytes + off;
  if (a.to_device) *dp = a.lcodes[i]; else a.lcodes[i] = *dp;
}

// I4 V plane: tokens (2p, 2p+1) share a device byte, dims (2jj, 2jj+1) share a logical byte.
// One thread per (plane, token pair, dim pair) owns the 2 device bytes and 2 logical bytes involved
// and transposes the 2x2 nibbles; tokens outside [t0, t0+n_rows) keep their device nibbles.
__global__ __launch_bounds__(256) void k_cache_copy_i4v(CopyArgs a) {
  const int p0 = a.t0 >> 1, p1 = (a.t0 + a.n_rows - 1) >> 1;      // inclusive pair range
  const int n_pairs = p1 - p0 + 1;
  const int half = a.rank / 2;
  const int64_t total = (int64_t)a.n_planes * n_pairs * half;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int jj = (int)(i % half);
  const int64_t r2 = i / half;
  const int pr = (int)(r2 % n_pairs) + p0;
  const int64_t ph = r2 / n_pairs;
  const size_t plane_bytes = (size_t)a.t_cap * half;
  int nib;
  uint8_t* d0 = a.dcodes + ph * plane_bytes + i4_v_offset(2 * pr, 2 * jj, &nib);       // dim 2jj:   (token even | token odd << 4)
  uint8_t* d1 = a.dcodes + ph * plane_bytes + i4_v_offset(2 * pr, 2 * jj + 1, &nib);   // dim 2jj+1
  uint8_t dv0 = *d0, dv1 = *d1;
  for (int k = 0; k < 2; k++) {
    const int t = 2 * pr + k;
    if (t < a.t0 || t >= a.t0 + a.n_rows) continue;
    uint8_t* lp = a.lcodes + ((size_t)ph * a.n_rows + (t - a.t0)) * half + jj;          // (dim 2jj | dim 2jj+1 << 4) of token t
    if (a.to_device) {
      const uint8_t lv = *lp;
      const uint8_t c0 = lv & 0xF, c1 = lv >> 4;
      dv0 = k ? (uint8_t)((dv0 & 0x0F) | (c0 << 4)) : (uint8_t)((dv0 & 0xF0) | c0);
      dv1 = k ? (uint8_t)((dv1 & 0x0F) | (c1 << 4)) : (uint8_t)((dv1 & 0xF0) | c1);
    } else {
      const uint8_t c0 = k ? (dv0 >> 4) : (dv0 & 0xF), c1 = k ? (dv1 >> 4) : (dv1 & 0xF);
      *lp = (uint8_t)(c0 | (c1 << 4));
    }
  }
  if (a.to_device) { *d0 = dv0; *d1 = dv1; }
}

__global__ __launch_bounds__(256) void k_cache_copy_meta(CopyArgs a) {
  const int per = a.dtype == WSVD_I4 ? 2 : 1;
  const int64_t total = (int64_t)a.n_planes * a.n_rows * per;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int k = (int)(i % per);
  const int64_t rowi = i / per;
  const int tr = (int)(rowi % a.n_rows);
  const int64_t ph = rowi / a.n_rows;
  uint16_t* dp = a.dmeta + ((size_t)ph * a.t_cap + a.t0 + tr) * per + k;
  if (a.to_device) *dp = a.lmeta[i]; else a.lmeta[i] = *dp;
}

hipError_t wsvd_launch_cache_copy(bool to_device, const wsvd_layer_desc& d, int plane, void* logical_codes,
                                  void* logical_meta, int t0, int n_rows, void* dev_codes, void* dev_meta, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  CopyArgs a;
  a.lcodes = (uint8_t*)logical_codes; a.lmeta = (uint16_t*)logical_meta;
  a.dcodes = (uint8_t*)dev_codes; a.dmeta = (uint16_t*)dev_meta;
  a.n_planes = d.batch * d.n_kv_heads; a.t_cap = d.t_cap; a.t0 = t0; a.n_rows = n_rows; a.rank = d.rank;
  a.dtype = d.latent_dtype; a.plane = plane; a.to_device = to_device ? 1 : 0;
  const int rb = d.latent_dtype == WSVD_F32 ? d.rank * 4 : d.latent_dtype == WSVD_BF16 ? d.rank * 2
               : d.latent_dtype == WSVD_I8 ? d.rank : d.rank / 2;
  if (d.latent_dtype == WSVD_I4 && plane == 1) {
    const int n_pairs = ((t0 + n_rows - 1) >> 1) - (t0 >> 1) + 1;
    int64_t total = (int64_t)a.n_planes * n_pairs * (d.rank / 2);
    hipLaunchKernelGGL(k_cache_copy_i4v, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
  } else {
    int64_t total = (int64_t)a.n_planes * n_rows * rb;
    hipLaunchKernelGGL(k_cache_copy_bytes, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (d.latent_dtype == WSVD_I8 || d.latent_dtype == WSVD_I4) {
    int64_t total = (int64_t)a.n_planes * n_rows * (d.latent_dtype == WSVD_I4 ? 2 : 1);
    hipLaunchKernelGGL(k_cache_copy_meta, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
    e = hipGetLastError();
  }
  return e;
}

// ---------------------------------------------------------------- streaming-read probe (measurement aid)
// What the memory system gives a kernel that does nothing but read: each workgroup streams one contiguous share of
// the buffer with 16-byte loads, four per thread in flight, and folds the data into a value that is (practically)
// never stored.  Benchmarks run it over the very buffers the attention streams, to put the attention's bytes per
// second next to the rate a pure reader reaches on the same data, launch for launch.
__global__ __launch_bounds__(512) void k_stream_read(const v4i* __restrict__ base, size_t n16, int* __restrict__ sink) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
  int acc = 0;
  for (size_t i = lo + threadIdx.x; i < hi; i += 4 * 512) {
    v4i v[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const size_t j = i + (size_t)u * 512;
      v[u] = __builtin_nontemporal_load(base + (j < hi ? j : hi - 1));
    }
#pragma unroll
    for (int u = 0; u < 4; u++) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  if (acc == 0x5A17C0DE && sink) *sink = acc;
}

hipError_t wsvd_launch_stream_read(const void* ptr, size_t bytes, int workgroups, int* sink, hipStream_t s) {
  if (bytes < 16 || workgroups < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_stream_read, dim3((unsigned)workgroups), dim3(512), 0, s, (const v4i*)ptr, bytes / 16, sink);
  return hipGetLastError();
}
