// Device-side helpers shared by the gfx950 kernels: storage formats, the latent quantisers,
// wave64 DPP reductions and the cache layouts declared in wsvd.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/wsvd.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf16 __attribute__((ext_vector_type(8)));
typedef _Float16 v8f16 __attribute__((ext_vector_type(8)));
typedef _Float16 v4f16 __attribute__((ext_vector_type(4)));

#define WSVD_DEV __device__ __forceinline__

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------- in-kernel timeline (profiling build only)
// Built with -DWSVD_TIMELINE, lane 0 of every wavefront writes the chip-wide 100 MHz wall clock into
// buf[(workgroup * 16 + wave) * 16 + slot] at the marked points; the product build compiles the marks out.
constexpr int kTimelineWaves = 16, kTimelineSlots = 16;
#ifdef WSVD_TIMELINE
#define WSVD_STAMP(buf, wg, wave, slot)                                                                          \
  do {                                                                                                           \
    if ((buf) && (threadIdx.x & 63) == 0)                                                                        \
      (buf)[((size_t)(wg) * kTimelineWaves + (wave)) * kTimelineSlots + (slot)] = (long long)wall_clock64();     \
  } while (0)
#else
#define WSVD_STAMP(buf, wg, wave, slot) do { } while (0)
#endif

// ---------------------------------------------------------------- matrix-core helpers
// 32x32 products of one wavefront.  Operand lane L holds row (column) L % 32 and the 8 (int8: 16) contraction
// indices starting at 8 (16) * (L / 32); accumulator lane L holds column L % 32, rows 8 (v / 4) + 4 (L / 32) + v % 4.
WSVD_DEV v16f mfma_bf16(v8bf16 a, v8bf16 b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
WSVD_DEV v16f mfma_f16(v8f16 a, v8f16 b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
WSVD_DEV v16i mfma_i8(v4i a, v4i b, v16i c) { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }

// 8 int8 codes (two dwords) -> 8 fp16 operand elements, exact.  A byte u = code + 128 placed under the high byte 0x64
// reads as the fp16 number 1024 + u; one byte permute builds two of them, one packed subtraction of 1152 ends it.
WSVD_DEV v8f16 codes_f16(int d0, int d1) {
  const uint32_t x0 = (uint32_t)d0 ^ 0x80808080u, x1 = (uint32_t)d1 ^ 0x80808080u;
  v4i r;
  r[0] = (int)__builtin_amdgcn_perm(0x64646464u, x0, 0x04010400u);
  r[1] = (int)__builtin_amdgcn_perm(0x64646464u, x0, 0x04030402u);
  r[2] = (int)__builtin_amdgcn_perm(0x64646464u, x1, 0x04010400u);
  r[3] = (int)__builtin_amdgcn_perm(0x64646464u, x1, 0x04030402u);
  return __builtin_bit_cast(v8f16, r) - (_Float16)1152;
}

// ---------------------------------------------------------------- storage formats
WSVD_DEV float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
WSVD_DEV uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
WSVD_DEV float f16_bits_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
WSVD_DEV uint16_t f32_to_f16_bits_rne(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// Load element idx of a tensor of dtype F32 / BF16 as float (I8 handled by the callers: it needs a scale).
WSVD_DEV float load_as_f32(const void* p, size_t idx, int dtype) {
  return dtype == WSVD_F32 ? ((const float*)p)[idx] : bf16_to_f32(((const uint16_t*)p)[idx]);
}

// ---------------------------------------------------------------- cross-workgroup hand-off
// Agent-scope relaxed accesses: the store is written through and the load bypasses non-coherent cache
// lines, so data handed from one workgroup to another (possibly on another XCD, behind another L2) needs
// no cache-wide write-back / invalidate.  Ordering comes from the barriers and waits around the ticket.
// Wait until every vector-memory operation this wave has issued is complete (for stores: acknowledged).  A
// workgroup barrier alone does not imply it: the barrier's workgroup-scope ordering needs no drain because the
// waves of a workgroup share their path to memory.  Hand-offs to OTHER workgroups (write-through stores, then a
// ticket or a flag) need the drain first.   Encoding: vmcnt = 0, expcnt and lgkmcnt left at their maxima.
WSVD_DEV void wait_vmem_done() { __builtin_amdgcn_s_waitcnt(0x0F70); }
WSVD_DEV void agent_store(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
WSVD_DEV float agent_load(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// ---------------------------------------------------------------- wave64 reductions (DPP)
template <int CTRL>
WSVD_DEV float dpp_mov_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
constexpr int kDppQuadSwap1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// After these four steps every lane of a 16-lane row holds the row's reduction.
WSVD_DEV float row16_max(float x) {
  x = fmaxf(x, dpp_mov_f<kDppQuadSwap1>(x));
  x = fmaxf(x, dpp_mov_f<kDppQuadSwap2>(x));
  x = fmaxf(x, dpp_mov_f<kDppRowHalfMirror>(x));
  x = fmaxf(x, dpp_mov_f<kDppRowMirror>(x));
  return x;
}
WSVD_DEV float row16_sum(float x) {
  x += dpp_mov_f<kDppQuadSwap1>(x);
  x += dpp_mov_f<kDppQuadSwap2>(x);
  x += dpp_mov_f<kDppRowHalfMirror>(x);
  x += dpp_mov_f<kDppRowMirror>(x);
  return x;
}
WSVD_DEV float lane_bcast(float x, int lane) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane)); }
WSVD_DEV float wave_max(float x) {
  x = row16_max(x);
  return fmaxf(fmaxf(lane_bcast(x, 0), lane_bcast(x, 16)), fmaxf(lane_bcast(x, 32), lane_bcast(x, 48)));
}
WSVD_DEV float wave_sum(float x) {
  x = row16_sum(x);
  return (lane_bcast(x, 0) + lane_bcast(x, 16)) + (lane_bcast(x, 32) + lane_bcast(x, 48));
}
// reductions over each half of the wave (lanes 0..31 and 32..63 separately); result valid in every lane of the half
WSVD_DEV float half_max(float x, int lane) {
  x = row16_max(x);
  float lo = fmaxf(lane_bcast(x, 0), lane_bcast(x, 16)), hi = fmaxf(lane_bcast(x, 32), lane_bcast(x, 48));
  return lane < 32 ? lo : hi;
}
WSVD_DEV float half_sum(float x, int lane) {
  x = row16_sum(x);
  float lo = lane_bcast(x, 0) + lane_bcast(x, 16), hi = lane_bcast(x, 32) + lane_bcast(x, 48);
  return lane < 32 ? lo : hi;
}
// maximum over groups of N adjacent lanes (N = 2,4,8,16); every lane of the group gets the result
template <int N>
WSVD_DEV float group_max(float x) {
  if (N >= 2) x = fmaxf(x, dpp_mov_f<kDppQuadSwap1>(x));
  if (N >= 4) x = fmaxf(x, dpp_mov_f<kDppQuadSwap2>(x));
  if (N >= 8) x = fmaxf(x, dpp_mov_f<kDppRowHalfMirror>(x));
  if (N >= 16) x = fmaxf(x, dpp_mov_f<kDppRowMirror>(x));
  return x;
}
// sum over groups of N adjacent lanes (N = 2,4,8,16); every lane of the group gets the result
template <int N>
WSVD_DEV float group_sum(float x) {
  if (N >= 2) x += dpp_mov_f<kDppQuadSwap1>(x);
  if (N >= 4) x += dpp_mov_f<kDppQuadSwap2>(x);
  if (N >= 8) x += dpp_mov_f<kDppRowHalfMirror>(x);
  if (N >= 16) x += dpp_mov_f<kDppRowMirror>(x);
  return x;
}

// ---------------------------------------------------------------- latent quantisers (rules in wsvd.h)
WSVD_DEV uint16_t guard_scale_f16(float s32) {
  uint16_t h = f32_to_f16_bits_rne(s32);
  if ((h & 0x7FFFu) == 0) h = 0x0001u;        // zero -> smallest subnormal 2^-24
  if ((h & 0x7FFFu) == 0x7C00u) h = 0x7BFFu;  // inf -> 65504
  return h;
}

// c: R fp32 values (registers or LDS).  Writes R int8 codes, returns the fp16 scale bits.
template <int R>
WSVD_DEV uint16_t quantize_row_i8(const float* c, int8_t* codes) {
  float a = 0.f;
#pragma unroll
  for (int j = 0; j < R; j++) a = fmaxf(a, fabsf(c[j]));
  uint16_t sh = 0x3C00u;  // 1.0
  if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
  float s = f16_bits_to_f32(sh);
#pragma unroll
  for (int j = 0; j < R; j++) {
    float v = __builtin_rintf(c[j] / s);
    v = fminf(fmaxf(v, -127.f), 127.f);
    codes[j] = (int8_t)(int)v;
  }
  return sh;
}

// Writes R codes in [0,15] (one per byte, unpacked), returns scale bits and zero-point bits.
template <int R>
WSVD_DEV void quantize_row_i4(const float* c, uint8_t* codes, uint16_t* scale_bits, uint16_t* zero_bits) {
  float lo = 0.f, hi = 0.f;
#pragma unroll
  for (int j = 0; j < R; j++) { lo = fminf(lo, c[j]); hi = fmaxf(hi, c[j]); }
  uint16_t sh = 0x3C00u;
  float z = 0.f;
  const bool flat = (hi == lo);
  if (!flat) sh = guard_scale_f16((hi - lo) / 15.0f);
  float s = f16_bits_to_f32(sh);
  if (!flat) z = fminf(fmaxf(__builtin_rintf(-lo / s), 0.f), 15.f);
  const int zi = (int)z;
#pragma unroll
  for (int j = 0; j < R; j++) {
    // clamp in float first so the int conversion cannot overflow
    float v = fminf(fmaxf(__builtin_rintf(c[j] / s), -64.f), 64.f);
    int q = (int)v + zi;
    q = q < 0 ? 0 : (q > 15 ? 15 : q);
    codes[j] = (uint8_t)q;
  }
  *scale_bits = sh;
  *zero_bits = f32_to_f16_bits_rne((float)zi);   // integer code 0..15, never -0
}

// ---------------------------------------------------------------- cache layouts (see wsvd.h)
WSVD_DEV int row_code_bytes(int rank, int latent_dtype) {
  return latent_dtype == WSVD_F32 ? rank * 4 : latent_dtype == WSVD_BF16 ? rank * 2 : latent_dtype == WSVD_I8 ? rank : rank / 2;
}
// byte offset, inside one (b, kv head) plane, of int8 element (token t, dim j)
WSVD_DEV size_t i8_k_offset(int t, int j, int rank) {
  return (size_t)(t >> 5) * (size_t)(32 * rank) + (size_t)(((((j >> 5) << 1) + ((j & 31) >> 4)) * 32 + (t & 31)) * 16 + (j & 15));
}
WSVD_DEV size_t i8_v_offset(int t, int j, int rank) {
  const int n = t & 31;
  return (size_t)(t >> 5) * (size_t)(32 * rank) + (size_t)(((((j >> 5) << 1) + (n >> 4)) * 32 + (j & 31)) * 16 + (n & 15));
}
// int4, rank 32: byte offset and nibble (0 = low) of element (token t, dim j)
WSVD_DEV size_t i4_k_offset(int t, int j, int* nib) {
  const int tt = t & 63, slot = tt >> 5, n = tt & 31;
  *nib = j & 1;
  return (size_t)(t >> 6) * 1024 + (size_t)((j >> 4) * 512 + n * 16 + slot * 8 + ((j & 15) >> 1));
}
WSVD_DEV size_t i4_v_offset(int t, int j, int* nib) {
  const int tt = t & 63;
  *nib = tt & 1;
  return (size_t)(t >> 6) * 1024 + (size_t)(((tt >> 5) * 32 + j) * 16 + ((tt & 31) >> 1));
}

// ---------------------------------------------------------------- packed down-projection factor
// Element (kv head, latent channel j, model dim e) of a packed A factor: blocks of 32 channels x 16 model dims stored
// as the 64-lane x 8-element image of a 32x32x16 matrix-core operand (lane = (e%16)/8 * 32 + j%32).
WSVD_DEV size_t a_packed_offset(int kv, int j, int e, int rank, int d_model) {
  const int tiles = (rank + 31) >> 5;
  return ((((size_t)(kv * tiles + (j >> 5)) * (size_t)(d_model >> 4) + (size_t)(e >> 4)) * 2 + ((e & 15) >> 3)) * 32 + (j & 31)) * 8 + (e & 7);
}

// ---------------------------------------------------------------- workspace layout (host + device)
// [0, kWsCounterInts*4): counters (zeroed by wsvd_set_workspace, self-resetting); then the attention's split words and the
// append's pushed words (8-byte {value, tag} words, cleared by their consumer: zero between launches); then the fp32
// partial sums of the sliced append kernels, which the decode step's projection launch uses for its slices too (followed
// by its one pending word per sequence); no invariant there: written before read.
// ints [0, 8192): unused; [8192, 12288): append tickets; [12288, 16000): fused-step row flags
// (2*Hkv, hold the epoch of the last step); [16000]: fused-step finished-workgroup counter.
constexpr int kWsCounterInts = 16384;
constexpr int kWsStepFlagsInt = 12288;
constexpr int kWsStepDoneInt = 16000;
