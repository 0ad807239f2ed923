// Pieces shared by the decode-attention kernels: parameters, work decomposition, query absorption
// (q~ = B_K q), the split merge and the B_V epilogue.
#pragma once
#include "wsvd_dev.h"

struct AttnParams {
  const void* q;             // [B,Hq,d] q_dtype
  const uint16_t* q_scale;   // fp16 [B] iff q_dtype == I8
  const void* BK;            // [Hkv,R,d] factor_dtype
  const void* BV;
  const uint8_t* k_codes;
  const uint8_t* v_codes;
  const uint16_t* k_meta;
  const uint16_t* v_meta;
  const int* seq_lens;
  float* out;                // [B,Hq,d] fp32
  float* partials;           // [B*Hq][n_chunks][R+2] fp32 (m, l, u[R]) in the log2 domain, un-normalised
  int* tickets;              // [B*Hkv]
  int B, Hq, Hkv, G, d, t_cap;
  int chunk_rows;            // rows of context per workgroup (multiple of 64)
  int n_chunks;              // grid extent along the context
  int q_dtype, factor_dtype;
  float c_scale;             // sm_scale * log2(e): scores live in the log2 domain
};

struct WorkItem {
  int b, kv, chunk, n, row_begin, row_end, n_splits;
  bool active;
};

// blockIdx.x -> (b, chunk, kv) with kv fastest: workgroups are dealt round-robin to the 8 XCDs, so with
// Hkv a multiple of 8 each XCD's L2 only ever sees the B factors of Hkv/8 heads.
WSVD_DEV WorkItem decode_work(const AttnParams& p) {
  WorkItem w;
  int id = blockIdx.x;
  w.kv = id % p.Hkv;
  id /= p.Hkv;
  w.chunk = id % p.n_chunks;
  w.b = id / p.n_chunks;
  w.n = p.seq_lens[w.b];
  w.n = w.n < 0 ? 0 : (w.n > p.t_cap ? p.t_cap : w.n);
  w.n_splits = (w.n + p.chunk_rows - 1) / p.chunk_rows;
  w.row_begin = w.chunk * p.chunk_rows;
  w.row_end = min(w.n, w.row_begin + p.chunk_rows);
  w.active = w.chunk < w.n_splits;
  return w;
}

// A sequence with no rows: its outputs are zeros (written by the chunk-0 workgroup).
WSVD_DEV void write_zero_outputs(const AttnParams& p, const WorkItem& w) {
  if (w.chunk != 0) return;
  for (int i = threadIdx.x; i < p.G * p.d; i += blockDim.x)
    p.out[((size_t)w.b * p.Hq + w.kv * p.G) * p.d + i] = 0.f;
}

WSVD_DEV float load_q(const AttnParams& p, size_t idx, float qs) {
  if (p.q_dtype == WSVD_I8) return (float)((const int8_t*)p.q)[idx] * qs;
  return load_as_f32(p.q, idx, p.q_dtype);
}

// q~[g][j] = c_scale * sum_c B_K[kv][j][c] * q[b, kv*G+g][c]   (query absorption; 256 threads).
// Ends with a __syncthreads.
template <int R>
WSVD_DEV void compute_qtilde(const AttnParams& p, const WorkItem& w, float* qts /* LDS [G][R] */) {
  constexpr int TPJ = 256 / R;            // threads cooperating on one latent dim
  const int tid = threadIdx.x;
  const int j = tid / TPJ, part = tid % TPJ;
  const int CP = p.d / TPJ;               // head-dim columns per thread
  const float qs = p.q_dtype == WSVD_I8 ? f16_bits_to_f32(p.q_scale[w.b]) : 1.f;
  const size_t brow = ((size_t)w.kv * R + j) * p.d + (size_t)part * CP;
  for (int g = 0; g < p.G; g++) {
    const size_t qrow = ((size_t)w.b * p.Hq + (size_t)w.kv * p.G + g) * p.d + (size_t)part * CP;
    float acc = 0.f;
    for (int c = 0; c < CP; c++) acc = fmaf(load_as_f32(p.BK, brow + c, p.factor_dtype), load_q(p, qrow + c, qs), acc);
    acc = group_sum<TPJ>(acc);
    if (part == 0) qts[g * R + j] = acc * p.c_scale;
  }
  __syncthreads();
}

// Tail of every attention kernel.  On entry Msh[g], Lsh[g], Ush[g*R+j] hold this workgroup's running
// max (log2 domain), sum and un-normalised latent-space accumulator, visible to all threads.
// If the sequence was split over several workgroups the partials go to the workspace and the last
// workgroup to arrive (ticket) merges them in split order; then out = (u / l) B_V.
template <int R>
WSVD_DEV void attn_tail(const AttnParams& p, const WorkItem& w, float* Msh, float* Lsh, float* Ush, int* flag_sh) {
  const int tid = threadIdx.x;
  const int G = p.G;
  if (w.n_splits > 1) {
    for (int i = tid; i < G * (R + 2); i += blockDim.x) {
      const int g = i / (R + 2), k = i % (R + 2);
      const float v = k == 0 ? Msh[g] : k == 1 ? Lsh[g] : Ush[g * R + (k - 2)];
      p.partials[(((size_t)w.b * p.Hq + w.kv * G + g) * p.n_chunks + w.chunk) * (R + 2) + k] = v;
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      int* t = p.tickets + (size_t)w.b * p.Hkv + w.kv;
      const int old = atomicAdd(t, 1);
      const int last = (old == w.n_splits - 1);
      if (last) atomicExch(t, 0);   // every other workgroup of this (b, kv) has already taken its ticket
      *flag_sh = last;
    }
    __syncthreads();
    if (!*flag_sh) return;
    __threadfence();
    for (int i = tid; i < G * R; i += blockDim.x) {
      const int g = i / R, j = i % R;
      const float* base = p.partials + (((size_t)w.b * p.Hq + w.kv * G + g) * p.n_chunks) * (R + 2);
      float M = -INFINITY;
      for (int c = 0; c < w.n_splits; c++) M = fmaxf(M, __builtin_nontemporal_load(base + (size_t)c * (R + 2)));
      float L = 0.f, U = 0.f;
      for (int c = 0; c < w.n_splits; c++) {
        const float* pc = base + (size_t)c * (R + 2);
        const float e = __builtin_amdgcn_exp2f(__builtin_nontemporal_load(pc) - M);
        L = fmaf(__builtin_nontemporal_load(pc + 1), e, L);
        U = fmaf(__builtin_nontemporal_load(pc + 2 + j), e, U);
      }
      Ush[i] = U;
      if (j == 0) { Lsh[g] = L; Msh[g] = M; }
    }
    __syncthreads();
  }
  // out[b, h, c] = sum_j (U[g][j] / L[g]) * B_V[kv][j][c]
  for (int i = tid; i < G * p.d; i += blockDim.x) {
    const int g = i / p.d, c = i % p.d;
    const float inv = 1.f / Lsh[g];
    float acc = 0.f;
#pragma unroll 8
    for (int j = 0; j < R; j++)
      acc = fmaf(Ush[g * R + j], load_as_f32(p.BV, ((size_t)w.kv * R + j) * p.d + c, p.factor_dtype), acc);
    p.out[((size_t)w.b * p.Hq + w.kv * G + g) * p.d + c] = acc * inv;
  }
}
