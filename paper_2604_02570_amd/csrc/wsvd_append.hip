// Latent append: c_K = x A_K[h], c_V = x A_V[h] for the new token of every sequence, rounded to the
// cache's storage format and written at row seq_lens[b] (decoding pipeline of Section 3.4).
//
// The contraction over d_model is split into ES slices so that enough workgroups stream the factors;
// slice partials go to the workspace and the last workgroup of a (plane, kv head) to arrive sums them
// in slice order (deterministic), quantises and stores.  The very last workgroup bumps seq_lens.
#include "wsvd_dev.h"
#include "wsvd_internal.h"

struct AppendParams {
  const void* x;             // [B,E]
  const uint16_t* x_scale;   // fp16 [B] iff x_dtype == I8
  const void* A[2];          // A_K, A_V [Hkv,E,R]
  uint8_t* codes[2];
  uint16_t* meta[2];
  int* seq_lens;
  float* partials;           // [2][Hkv][ES][B][R]
  int* tickets;              // [2*Hkv] per-plane tickets, then [1] global ticket
  int* err_word;
  int B, E, Hkv, t_cap, ES, ESL;
  int x_dtype, factor_dtype, latent_dtype;
};

constexpr int kAppendBB = 8;       // batch rows per pass
constexpr int kAppendMaxESL = 256; // d_model slice per workgroup

WSVD_DEV float load_x(const AppendParams& p, int b, int e) {
  const size_t idx = (size_t)b * p.E + e;
  if (p.x_dtype == WSVD_I8) return (float)((const int8_t*)p.x)[idx] * f16_bits_to_f32(p.x_scale[b]);
  return load_as_f32(p.x, idx, p.x_dtype);
}

// Store one latent row (fp32 values in c[0..R)) of (b, kv) at row t of plane `pl`.
template <int R>
WSVD_DEV void store_row(const AppendParams& p, int pl, int b, int kv, int t, const float* c) {
  const size_t ph = (size_t)b * p.Hkv + kv;
  if (p.latent_dtype == WSVD_F32) {
    float* dst = (float*)p.codes[pl] + (ph * p.t_cap + t) * R;
    for (int j = 0; j < R; j++) dst[j] = c[j];
  } else if (p.latent_dtype == WSVD_BF16) {
    uint16_t* dst = (uint16_t*)p.codes[pl] + (ph * p.t_cap + t) * R;
    for (int j = 0; j < R; j++) dst[j] = f32_to_bf16_rne(c[j]);
  } else if (p.latent_dtype == WSVD_I8) {
    float v[R];
    int8_t q[R];
#pragma unroll
    for (int j = 0; j < R; j++) v[j] = c[j];
    const uint16_t sh = quantize_row_i8<R>(v, q);
    uint8_t* plane = p.codes[pl] + ph * (size_t)p.t_cap * R;
    for (int j = 0; j < R; j++) plane[pl == 0 ? i8_k_offset(t, j, R) : i8_v_offset(t, j, R)] = (uint8_t)q[j];
    p.meta[pl][ph * p.t_cap + t] = sh;
  } else {  // I4, R == 32
    float v[R];
    uint8_t q[R];
#pragma unroll
    for (int j = 0; j < R; j++) v[j] = c[j];
    uint16_t sh, zh;
    quantize_row_i4<R>(v, q, &sh, &zh);
    uint8_t* plane = p.codes[pl] + ph * (size_t)p.t_cap * (R / 2);
    if (pl == 0) {
      for (int j = 0; j < R; j += 2) { int nib; plane[i4_k_offset(t, j, &nib)] = (uint8_t)(q[j] | (q[j + 1] << 4)); }
    } else {
      // tokens (t, t^1) share each byte; the other token was (or will be) written by a different launch
      for (int j = 0; j < R; j++) {
        int nib;
        uint8_t* bp = plane + i4_v_offset(t, j, &nib);
        const uint8_t old = *bp;
        *bp = nib ? (uint8_t)((old & 0x0F) | (q[j] << 4)) : (uint8_t)((old & 0xF0) | q[j]);
      }
    }
    p.meta[pl][(ph * p.t_cap + t) * 2] = sh;
    p.meta[pl][(ph * p.t_cap + t) * 2 + 1] = zh;
  }
}

template <int R, int FESZ>
__global__ __launch_bounds__(256) void k_append(AppendParams p) {
  constexpr int EL = 256 / R;                 // threads along d_model per latent dim
  constexpr int NA = kAppendMaxESL / EL;      // factor elements per thread (one d_model slice, one latent dim)
  __shared__ __attribute__((aligned(16))) float xs[kAppendMaxESL][kAppendBB];
  __shared__ float red[EL][kAppendBB][R];
  __shared__ float crow[64][R + 1];
  __shared__ int flag_sh;

  int id = blockIdx.x;
  const int s = id % p.ES; id /= p.ES;
  const int kv = id % p.Hkv;
  const int pl = id / p.Hkv;
  const int tid = threadIdx.x, j = tid % R, el = tid / R;
  const int e0 = s * p.ESL;
  float* part = p.partials + ((((size_t)pl * p.Hkv + kv) * p.ES + s) * p.B) * R;

  // this thread's slice of the factor: read once (all loads in flight together), reused for every batch row
  float a[NA];
#pragma unroll
  for (int i = 0; i < NA; i++) {
    const int e = el + i * EL;
    const size_t idx = ((size_t)kv * p.E + e0 + e) * R + j;
    a[i] = 0.f;
    if (e < p.ESL) a[i] = FESZ == 4 ? ((const float*)p.A[pl])[idx] : bf16_to_f32(((const uint16_t*)p.A[pl])[idx]);
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
  // ---- ticket of this (plane, kv head).  Partials travel as agent-scope accesses (no cache-wide fences);
  // the barrier makes sure every thread's stores have completed before the ticket is taken.
  __syncthreads();
  if (tid == 0) {
    int* t = p.tickets + pl * p.Hkv + kv;
    const int old = __hip_atomic_fetch_add(t, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == p.ES - 1);
    if (last) __hip_atomic_store(t, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    flag_sh = last;
  }
  __syncthreads();
  if (!flag_sh) return;
  const float* pbase = p.partials + (((size_t)pl * p.Hkv + kv) * p.ES) * p.B * R;
  for (int b0 = 0; b0 < p.B; b0 += 64) {
    const int nb = min(64, p.B - b0);
    __syncthreads();
    for (int i = tid; i < nb * R; i += 256) {
      const int bb = i / R, jj = i % R;
      float sum = 0.f;
      for (int k = 0; k < p.ES; k++) sum += agent_load(pbase + ((size_t)k * p.B + b0 + bb) * R + jj);
      crow[bb][jj] = sum;
    }
    __syncthreads();
    if (tid < nb) {
      const int b = b0 + tid;
      const int n = p.seq_lens[b];
      if (n >= 0 && n < p.t_cap) store_row<R>(p, pl, b, kv, n, crow[tid]);
    }
  }
  // ---- global ticket: the last finisher advances the sequence lengths (it only touches seq_lens, which no
  // other workgroup writes; the rows stored above are consumed by later launches)
  __syncthreads();
  if (tid == 0) {
    int* t = p.tickets + 2 * p.Hkv;
    const int old = __hip_atomic_fetch_add(t, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == 2 * p.Hkv - 1);
    if (last) __hip_atomic_store(t, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    flag_sh = last;
  }
  __syncthreads();
  if (!flag_sh) return;
  for (int b = tid; b < p.B; b += 256) {
    const int n = p.seq_lens[b];
    if (n >= 0 && n < p.t_cap) p.seq_lens[b] = n + 1;
    else atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
  }
}

int wsvd_append_esplits(const wsvd_layer_desc& d) {
  int esl = kAppendMaxESL;
  while (esl > 1 && d.d_model % esl != 0) esl >>= 1;
  return d.d_model / esl;
}
size_t wsvd_append_partial_floats(const wsvd_layer_desc& d) {
  return (size_t)2 * d.n_kv_heads * wsvd_append_esplits(d) * d.batch * d.rank;
}

hipError_t wsvd_launch_append(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale,
                              const void* A_K, const void* A_V, const wsvd_cache& cache, hipStream_t s) {
  AppendParams p;
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
  dim3 grid((unsigned)(p.ES * p.Hkv * 2)), block(256);
  const bool f32 = d.factor_dtype == WSVD_F32;
  switch (d.rank) {
    case 16: if (f32) hipLaunchKernelGGL((k_append<16, 4>), grid, block, 0, s, p); else hipLaunchKernelGGL((k_append<16, 2>), grid, block, 0, s, p); break;
    case 32: if (f32) hipLaunchKernelGGL((k_append<32, 4>), grid, block, 0, s, p); else hipLaunchKernelGGL((k_append<32, 2>), grid, block, 0, s, p); break;
    case 64: if (f32) hipLaunchKernelGGL((k_append<64, 4>), grid, block, 0, s, p); else hipLaunchKernelGGL((k_append<64, 2>), grid, block, 0, s, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
