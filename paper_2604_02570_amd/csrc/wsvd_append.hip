// Latent append: c_K = x A_K[h], c_V = x A_V[h] for the new token of every sequence, rounded to the
// cache's storage format and written at row seq_lens[b] (decoding pipeline of Section 3.4).
//
// The factors arrive PACKED (wsvd_pack_factor_a): blocks of 32 latent channels x 16 model dims stored as the
// register image of a 32x32x16 matrix-core operand, so a wavefront's 64 x 16-byte load is one contiguous KiB
// and is the operand itself.
// The contraction over d_model is split into ES slices so that enough workgroups stream the factors;
// slice partials go to the workspace and the last workgroup of a (plane, kv head) to arrive sums them
// in slice order (deterministic), quantises and stores.  The very last workgroup bumps seq_lens.
//   bf16 factors and bf16 x: V_MFMA_F32_32X32X16_BF16, D[latent channel][sequence];
//   anything else (the all-fp32 configuration): vector ALU.
#include "wsvd_dev.h"
#include "wsvd_append_body.h"

// ---------------------------------------------------------------- vector-ALU path (any dtype)
template <int R, int FESZ>
__global__ __launch_bounds__(256) void k_append_valu(AppendParams p) {
  constexpr int EL = 256 / R;                 // threads along d_model per latent channel
  constexpr int NA = kAppendMaxESL / EL;      // factor elements per thread
  __shared__ __attribute__((aligned(16))) float xs[kAppendMaxESL][kAppendBB];
  __shared__ float red[EL][kAppendBB][R];
  __shared__ float crow[64][R + 1];
  __shared__ int flag_sh;
  __shared__ int n_sh[kAppendMaxB];

  append_read_lens(p, n_sh);
  int s, kv, pl;
  append_coords(p, blockIdx.x, s, kv, pl);
  const int tid = threadIdx.x, j = tid % R, el = tid / R;
  const int e0 = s * p.ESL;
  float* part = p.partials + ((((size_t)pl * p.Hkv + kv) * p.ES + s) * p.B) * R;

  // this thread's slice of channel j: read once (all loads in flight together), reused for every sequence
  float a[NA];
#pragma unroll
  for (int i = 0; i < NA; i++) {
    const int e = min(el + i * EL, p.ESL - 1);
    const size_t idx = a_packed_offset(kv, j, e0 + e, R, p.E);
    a[i] = FESZ == 4 ? ((const float*)p.A[pl])[idx] : bf16_to_f32(((const uint16_t*)p.A[pl])[idx]);
  }

  for (int b0 = 0; b0 < p.B; b0 += kAppendBB) {
    const int nb = min(kAppendBB, p.B - b0);
    __syncthreads();
    for (int i = tid; i < kAppendBB * p.ESL; i += 256) {
      const int bb = i / p.ESL, e = i % p.ESL;
      xs[e][bb] = bb < nb ? load_x(p, b0 + bb, e0 + e) : 0.f;
    }
    __syncthreads();
    float acc[kAppendBB];
#pragma unroll
    for (int bb = 0; bb < kAppendBB; bb++) acc[bb] = 0.f;
#pragma unroll
    for (int i = 0; i < NA; i++) {
      const int e = el + i * EL;
      if (e < p.ESL) {
        const v4f x0 = *(const v4f*)&xs[e][0], x1 = *(const v4f*)&xs[e][4];
#pragma unroll
        for (int bb = 0; bb < 4; bb++) { acc[bb] = fmaf(x0[bb], a[i], acc[bb]); acc[4 + bb] = fmaf(x1[bb], a[i], acc[4 + bb]); }
      }
    }
#pragma unroll
    for (int bb = 0; bb < kAppendBB; bb++) red[el][bb][j] = acc[bb];
    __syncthreads();
    for (int i = tid; i < nb * R; i += 256) {
      const int bb = i / R, jj = i % R;
      float sum = 0.f;
      for (int k = 0; k < EL; k++) sum += red[k][bb][jj];
      agent_store(&part[(size_t)(b0 + bb) * R + jj], sum);
    }
  }
  append_finish<R>(p, pl, kv, crow, &flag_sh, n_sh);
}

// ---------------------------------------------------------------- factor packing (set-up time)
__global__ __launch_bounds__(256) void k_pack_factor_a(const void* __restrict__ src, void* __restrict__ dst, int Hkv, int E, int R, int esz) {
  const int tiles = (R + 31) >> 5;
  const size_t total = (size_t)Hkv * tiles * 32 * E;       // packed elements, channels padded to a multiple of 32
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  // decode the packed position
  const int e7 = (int)(i & 7); size_t r = i >> 3;
  const int c = (int)(r & 31); r >>= 5;
  const int g = (int)(r & 1); r >>= 1;
  const int eb = (int)(r % (size_t)(E >> 4)); r /= (size_t)(E >> 4);
  const int tile = (int)(r % tiles); const int kv = (int)(r / tiles);
  const int j = tile * 32 + c, e = eb * 16 + g * 8 + e7;
  const size_t sidx = ((size_t)kv * E + e) * R + j;
  if (esz == 4) ((uint32_t*)dst)[i] = j < R ? ((const uint32_t*)src)[sidx] : 0u;
  else ((uint16_t*)dst)[i] = j < R ? ((const uint16_t*)src)[sidx] : (uint16_t)0;
}

hipError_t wsvd_launch_pack_factor_a(const wsvd_layer_desc& d, const void* src, void* dst, hipStream_t s) {
  const size_t total = (size_t)d.n_kv_heads * ((d.rank + 31) / 32) * 32 * d.d_model;
  hipLaunchKernelGGL(k_pack_factor_a, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, src, dst, d.n_kv_heads, d.d_model,
                     d.rank, d.factor_dtype == WSVD_F32 ? 4 : 2);
  return hipGetLastError();
}

// d_model slices per (plane, kv head).
// One CU cannot pull more than a few tens of GB/s on its own, so the factor stream has to be spread over all of
// them: the MFMA path aims at about one workgroup per CU (256) and merges the slices through the ticket.
// The vector-ALU path keeps slices of at most 256 elements (its LDS staging size).
int g_append_mode = 0;   // tuning: 0 = automatic, n > 0 = force n slices (MFMA path)
static bool append_mfma_path(const wsvd_layer_desc& d) { return d.factor_dtype == WSVD_BF16 && d.x_dtype == WSVD_BF16; }
int wsvd_append_esplits(const wsvd_layer_desc& d) {
  if (!append_mfma_path(d)) {
    int esl = kAppendMaxESL;
    while (esl > 64 && d.d_model % esl != 0) esl >>= 1;
    return d.d_model / esl;
  }
  const int units = d.d_model / 64;                              // slices are multiples of 64 elements
  int want = g_append_mode > 0 ? g_append_mode : 256 / (2 * d.n_kv_heads);
  if (want < 1) want = 1;
  // smallest slice count >= want whose slices fit the kernel's LDS staging; else the largest count that exists
  int es = units;
  for (int c = 1; c <= units; c++) {
    if (units % c != 0 || d.d_model / c > kAppendMfmaESL) continue;
    es = c;
    if (c >= want) break;
  }
  return es;
}
size_t wsvd_append_partial_floats(const wsvd_layer_desc& d) {
  return (size_t)2 * d.n_kv_heads * wsvd_append_esplits(d) * d.batch * d.rank;
}

void wsvd_append_params(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale, const void* A_K,
                        const void* A_V, const wsvd_cache& cache, AppendParams& p) {
  p = AppendParams{};
  p.x = x; p.x_scale = (const uint16_t*)x_scale;
  p.A[0] = A_K; p.A[1] = A_V;
  p.codes[0] = (uint8_t*)cache.k_codes; p.codes[1] = (uint8_t*)cache.v_codes;
  p.meta[0] = (uint16_t*)cache.k_meta; p.meta[1] = (uint16_t*)cache.v_meta;
  p.seq_lens = cache.seq_lens;
  p.tickets = (int*)ctx->ws + kWsCounterInts / 2;
  p.partials = (float*)((char*)ctx->ws + (size_t)kWsCounterInts * 4);
  p.err_word = ctx->err_word;
  p.B = d.batch; p.E = d.d_model; p.Hkv = d.n_kv_heads; p.t_cap = d.t_cap;
  p.ES = wsvd_append_esplits(d); p.ESL = d.d_model / p.ES;
  p.x_dtype = d.x_dtype; p.factor_dtype = d.factor_dtype; p.latent_dtype = d.latent_dtype;
  p.one_seq = -1;
}

// waves per workgroup of the MFMA path: each wave gets a multiple of 16 elements, at least 64; up to 16 waves
// (rank 64: 8, register budget)
int wsvd_append_mfma_waves(const wsvd_layer_desc& d) {
  const int esl = d.d_model / wsvd_append_esplits(d);
  int nw = d.rank == 64 ? 8 : 16;
  while (nw > 4 && ((esl / nw) % 16 != 0 || esl / nw < 64)) nw >>= 1;
  return nw;
}
bool wsvd_append_uses_mfma(const wsvd_layer_desc& d) { return append_mfma_path(d); }

hipError_t wsvd_launch_append(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale,
                              const void* A_K, const void* A_V, const wsvd_cache& cache, hipStream_t s, int one_seq) {
  AppendParams p;
  wsvd_append_params(ctx, d, x, x_scale, A_K, A_V, cache, p);
  p.one_seq = one_seq;
  if (d.d_model % 64 != 0 || d.batch > kAppendMaxB) return hipErrorInvalidValue;
  dim3 grid((unsigned)(p.ES * p.Hkv * 2));
  const bool f32 = d.factor_dtype == WSVD_F32;
  if (append_mfma_path(d)) {
    int nw = wsvd_append_mfma_waves(d);
    if (d.batch > 32) {
      // two groups of 32 sequences per pass over the factors; the second set of accumulators needs the register
      // budget of a workgroup of at most 8 waves
      if (nw > 8) nw = 8;
      dim3 block((unsigned)(nw * 64));
      switch (d.rank) {
        case 16: hipLaunchKernelGGL((k_append_mfma<16, 512, 2>), grid, block, 0, s, p); break;
        case 32: hipLaunchKernelGGL((k_append_mfma<32, 512, 2>), grid, block, 0, s, p); break;
        case 64: hipLaunchKernelGGL((k_append_mfma<64, 512, 2>), grid, block, 0, s, p); break;
        default: return hipErrorInvalidValue;
      }
      return hipGetLastError();
    }
    dim3 block((unsigned)(nw * 64));
    switch (d.rank) {
      case 16: hipLaunchKernelGGL((k_append_mfma<16, 1024, 1>), grid, block, 0, s, p); break;
      case 32: hipLaunchKernelGGL((k_append_mfma<32, 1024, 1>), grid, block, 0, s, p); break;
      case 64: hipLaunchKernelGGL((k_append_mfma<64, 512, 1>), grid, block, 0, s, p); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  dim3 block(256);
  switch (d.rank) {
    case 16: if (f32) hipLaunchKernelGGL((k_append_valu<16, 4>), grid, block, 0, s, p); else hipLaunchKernelGGL((k_append_valu<16, 2>), grid, block, 0, s, p); break;
    case 32: if (f32) hipLaunchKernelGGL((k_append_valu<32, 4>), grid, block, 0, s, p); else hipLaunchKernelGGL((k_append_valu<32, 2>), grid, block, 0, s, p); break;
    case 64: if (f32) hipLaunchKernelGGL((k_append_valu<64, 4>), grid, block, 0, s, p); else hipLaunchKernelGGL((k_append_valu<64, 2>), grid, block, 0, s, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------- store of latents computed elsewhere
// The quantise-and-store half of the append for callers that produce the latents with another GEMM (the
// int4-weight / int8-activation projection of the quantised setting, Section 4.2).  One workgroup per sequence:
// it reads the sequence's length once, stores the 2*Hkv rows with R lanes per row and then advances the length,
// so no cross-workgroup ordering is needed.
template <int R>
__global__ __launch_bounds__(1024) void k_latent_store(AppendParams p, const float* __restrict__ cK,
                                                       const float* __restrict__ cV, long ld) {
  const int b = blockIdx.x;
  const int total = 2 * p.Hkv * R;     // a multiple of 64 whenever the latents are quantised (R >= 32)
  // every thread reads the length itself (one broadcast load) together with its first latent: one round trip
  const int n = __hip_atomic_load(p.seq_lens + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const int i0 = min((int)threadIdx.x, total - 1);
  float c = ((i0 / R) / p.Hkv ? cV : cK)[(size_t)b * ld + ((i0 / R) % p.Hkv) * R + i0 % R];
  if (n < 0 || n >= p.t_cap) {
    if (threadIdx.x == 0) atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
    return;
  }
  for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
    const int row = idx / R, j = idx % R;
    const int pl = row / p.Hkv, kv = row % p.Hkv;
    if (idx != (int)threadIdx.x) c = (pl ? cV : cK)[(size_t)b * ld + kv * R + j];
    store_row_lanes<R>(p, pl, b, kv, n, j, c);
  }
  __syncthreads();     // every thread has consumed the old length
  if (threadIdx.x == 0) p.seq_lens[b] = n + 1;
}

hipError_t wsvd_launch_latent_store(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const float* cK, const float* cV,
                                    int64_t ld, const wsvd_cache& cache, hipStream_t s) {
  AppendParams p = {};
  p.codes[0] = (uint8_t*)cache.k_codes; p.codes[1] = (uint8_t*)cache.v_codes;
  p.meta[0] = (uint16_t*)cache.k_meta; p.meta[1] = (uint16_t*)cache.v_meta;
  p.seq_lens = cache.seq_lens;
  p.err_word = ctx->err_word;
  p.B = d.batch; p.E = d.d_model; p.Hkv = d.n_kv_heads; p.t_cap = d.t_cap;
  p.latent_dtype = d.latent_dtype;
  const int total = 2 * d.n_kv_heads * d.rank;
  int threads = (total + 63) / 64 * 64;
  if (threads > 1024) threads = 1024;
  dim3 grid((unsigned)d.batch), block((unsigned)threads);
  switch (d.rank) {
    case 16: hipLaunchKernelGGL((k_latent_store<16>), grid, block, 0, s, p, cK, cV, (long)ld); break;
    case 32: hipLaunchKernelGGL((k_latent_store<32>), grid, block, 0, s, p, cK, cV, (long)ld); break;
    case 64: hipLaunchKernelGGL((k_latent_store<64>), grid, block, 0, s, p, cK, cV, (long)ld); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
