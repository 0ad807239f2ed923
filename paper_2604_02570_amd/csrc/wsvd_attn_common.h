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
  unsigned long long* partials;   // [B*Hq][n_chunks][R+2] pushed words {fp32 value, tag} of (m, l, u[R]), log2 domain, un-normalised
  int* tickets;              // [B*Hkv] (the fused decode step's counters)
  int B, Hq, Hkv, G, d, t_cap;
  int chunk_rows;            // rows of context per workgroup (multiple of 64)
  int n_chunks;              // grid extent along the context
  int q_dtype, factor_dtype;
  float c_scale;             // sm_scale * log2(e): scores live in the log2 domain
  int* err_word;             // device status word of the context
  // fused decode step only: the append workgroups of the same launch publish row seq_lens[b] of kv head h's K / V
  // plane by setting flags[h] / flags[Hkv + h] to epoch
  const int* flags;
  int epoch;
  // latent-query / latent-output variant only: q is the Q latent [B,Hq,rq] fp32, qk_fold the per-head matrices
  // B_Q B_K^T [Hq,rq,R] fp32, out is [B,Hq,R]
  const float* qk_fold;
  int rq;
  int out_dim;               // floats per (sequence, head) of out: d, or R for the latent-output variant
  // several query tokens per sequence (prefill / multi-token decode) only: G = nq * Gr query slots per kv head, slot
  // s = token s / Gr, head s % Gr; token i sits at row seq_lens - n_after - nq + i and sees the rows up to its own
  int nq, Gr, n_after;
  long long* timeline;       // profiling build: stamp buffer (see WSVD_STAMP), else null
  // store-and-attend variant only: the new token's fp32 latents [B][new_ld] (kv head h at h * R), the per-sequence
  // counters of finished workgroups, the lengths to advance
  const float* new_k;
  const float* new_v;
  long new_ld;
  int* done;
  int* seq_lens_rw;
  // paged cache only (else block_table is null): k_codes / v_codes / k_meta / v_meta are pools of n_pages pages, a page
  // = page_rows rows of every kv head; block_table [B][max_pages]
  const int* block_table;
  int page_rows, max_pages, n_pages;
  // a launch that covers only some of a kv head's query heads (groups larger than a kernel holds run as several
  // launches): the first query head of kv head h is h * Gmem + g0 in q and out (0 / 0: Gmem = G, g0 = 0)
  int Gmem, g0;
  // deferred-row variant only (the decode step's second launch): the step's projection launch has left the new token's
  // latents as n_parts partial sums, new_k / new_v [part][B][new_ld] fp32 with part_stride floats between parts, has
  // advanced the lengths already and set pending[b] != 0 for every sequence whose last row is still to be written
  const int* pending;
  int n_parts;
  long part_stride;
  int out_bf16;              // out holds bf16 (round to nearest even) instead of fp32; never for the latent-space output
};

// element idx (pair idx, idx + 1) of the output, in the layer's output format
WSVD_DEV void out_put(const AttnParams& p, size_t idx, float v) {
  if (p.out_bf16) ((uint16_t*)p.out)[idx] = f32_to_bf16_rne(v);
  else p.out[idx] = v;
}
WSVD_DEV void out_put2(const AttnParams& p, size_t idx, float a, float b) {      // idx even
  if (p.out_bf16) *(uint32_t*)((uint16_t*)p.out + idx) = (uint32_t)f32_to_bf16_rne(a) | ((uint32_t)f32_to_bf16_rne(b) << 16);
  else { float2 r; r.x = a; r.y = b; *(float2*)&p.out[idx] = r; }
}

// first query head (row of q / out) of kv head `kv` in this launch
WSVD_DEV size_t first_head(const AttnParams& p, int kv) { return (size_t)kv * (p.Gmem ? p.Gmem : p.G) + p.g0; }

struct WorkItem {
  int b, kv, chunk, n, row_begin, row_end, n_splits;
  bool active;
};

// Grid = (Hkv, n_chunks, B): blockIdx.x = kv head, .y = context chunk, .z = sequence.  The linear workgroup id
// (x fastest) is dealt round-robin to the 8 XCDs, so with Hkv a multiple of 8 each XCD's L2 only ever sees the
// B factors of Hkv/8 heads.  No integer division on the way to the first load.
WSVD_DEV WorkItem decode_work(const AttnParams& p, int n_raw, int kv, int chunk, int b) {
  WorkItem w;
  w.kv = kv;
  w.chunk = chunk;
  w.b = b;
  w.n = n_raw < 0 ? 0 : (n_raw > p.t_cap ? p.t_cap : n_raw);
  w.n_splits = (w.n + p.chunk_rows - 1) / p.chunk_rows;
  w.row_begin = w.chunk * p.chunk_rows;
  w.row_end = min(w.n, w.row_begin + p.chunk_rows);
  w.active = w.chunk < w.n_splits;
  // a sequence longer than the caller's bound: the grid does not cover its tail.  Reported, never silently truncated.
  if (w.n > p.n_chunks * p.chunk_rows && chunk == 0 && threadIdx.x == 0) atomicExch(p.err_word, (int)WSVD_E_SHAPE);
  return w;
}
WSVD_DEV WorkItem decode_work(const AttnParams& p, int n_raw) { return decode_work(p, n_raw, blockIdx.x, blockIdx.y, blockIdx.z); }

// A sequence with no rows: its outputs are zeros (written by the chunk-0 workgroup).
WSVD_DEV void write_zero_outputs(const AttnParams& p, const WorkItem& w) {
  if (w.chunk != 0) return;
  for (int i = threadIdx.x; i < p.G * p.out_dim; i += blockDim.x)
    out_put(p, ((size_t)w.b * p.Hq + first_head(p, w.kv)) * p.out_dim + i, 0.f);
}

// ---- staging of the per-head factors into LDS.
// B_K[kv] and B_V[kv] are contiguous R*d blocks.  All global loads are issued first (predicated, fully
// unrolled) and committed to LDS later, so the caller can put other loads in flight in between and a
// single wait covers everything.
template <int MAXIT>
struct StageRegs { v4i v[MAXIT]; };

template <int MAXIT>
WSVD_DEV void stage_issue(StageRegs<MAXIT>& r, const void* src, int n16) {
  // Unconditional loads (index clamped): a load under a branch would force every later wait to drain the whole
  // queue, tile prefetches included, because the wait-count bookkeeping is conservative across control flow.
#pragma unroll
  for (int it = 0; it < MAXIT; it++) {
    const int idx = min(it * (int)blockDim.x + (int)threadIdx.x, n16 - 1);
    r.v[it] = ((const v4i*)src)[idx];
  }
}
template <int MAXIT>
WSVD_DEV void stage_commit(const StageRegs<MAXIT>& r, void* lds, int n16) {
#pragma unroll
  for (int it = 0; it < MAXIT; it++) {
    const int idx = it * (int)blockDim.x + (int)threadIdx.x;
    if (idx < n16) ((v4i*)lds)[idx] = r.v[it];
  }
}

// queries of the G heads of kv head `kv` of sequence `b` -> LDS floats [G][d].  Split into issue (global loads
// into registers) and commit (LDS stores) so that other loads can be put in flight in between.  G*d <= 256*N
// and the workgroup has at least 256 threads.
// The issue phase only loads raw bits (no arithmetic on them), so it never waits.
template <int N>
struct QRegsT { uint32_t raw[N]; };
using QRegs = QRegsT<2>;
template <int N>
WSVD_DEV void q_issue(const AttnParams& p, int b, int kv, QRegsT<N>& r) {
  // one unconditional dword load per element: the aligned dword that contains it (4 int8, 2 bf16 or 1 fp32)
  const size_t base = ((size_t)b * p.Hq + first_head(p, kv)) * p.d;
  const int sh = p.q_dtype == WSVD_I8 ? 2 : p.q_dtype == WSVD_BF16 ? 1 : 0;
  const int n = p.G * p.d;
#pragma unroll
  for (int it = 0; it < N; it++) {
    const int i = min(it * 256 + (int)(threadIdx.x & 255), n - 1);
    r.raw[it] = ((const uint32_t*)p.q)[(base + i) >> sh];
  }
}
// fp16 scale of sequence b's int8 query through a scalar dword load (the buffer is 4-byte aligned and padded)
// Two-step so that the scalar load can be issued at the very top of a kernel and consumed late.
WSVD_DEV uint32_t q_scale_raw(const AttnParams& p, int b) {
  return p.q_dtype == WSVD_I8 ? ((const uint32_t*)p.q_scale)[b >> 1] : 0u;
}
WSVD_DEV float q_scale_value(const AttnParams& p, int b, uint32_t wraw) {
  if (p.q_dtype != WSVD_I8) return 1.f;
  return f16_bits_to_f32((uint16_t)((b & 1) ? (wraw >> 16) : (wraw & 0xFFFFu)));
}
template <int N>
WSVD_DEV void q_commit(const AttnParams& p, const QRegsT<N>& r, float qs, float* q_lds) {
  const int n = p.G * p.d;
#pragma unroll
  for (int it = 0; it < N; it++) {
    const int i = it * 256 + (int)threadIdx.x;
    if (threadIdx.x < 256 && i < n) {
      // (b*Hq + kv*G)*d is a multiple of 64, so element i sits at position i % (4 >> ...) of its dword
      float v;
      if (p.q_dtype == WSVD_I8) v = (float)(int8_t)(r.raw[it] >> ((i & 3) * 8)) * qs;
      else if (p.q_dtype == WSVD_BF16) v = __uint_as_float((i & 1) ? (r.raw[it] & 0xFFFF0000u) : (r.raw[it] << 16));
      else v = __uint_as_float(r.raw[it]);
      q_lds[i] = v;
    }
  }
}

// 8 consecutive factor elements from LDS as float
template <int ESZ>
WSVD_DEV void lds_load8(const void* lds, int idx, float* f) {
  if (ESZ == 4) {
    const v4f a = *(const v4f*)((const float*)lds + idx), b = *(const v4f*)((const float*)lds + idx + 4);
#pragma unroll
    for (int i = 0; i < 4; i++) { f[i] = a[i]; f[4 + i] = b[i]; }
  } else {
    const v4i raw = *(const v4i*)((const uint16_t*)lds + idx);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      f[2 * i] = __uint_as_float((uint32_t)raw[i] << 16);
      f[2 * i + 1] = __uint_as_float((uint32_t)raw[i] & 0xFFFF0000u);
    }
  }
}

// q~[g][j] = c_scale * sum_c B_K[kv][j][c] * q[b, kv*G+g][c]   (query absorption; whole workgroup, any multiple of 64 threads).
// bk_lds holds B_K[kv] (R x d, element size ESZ); q_lds [G][d] floats.  Work is split into chunks of 8
// columns: chunk id -> (row j, column block); the d/8 lanes of a row are adjacent.  Ends with a barrier.
template <int R, int ESZ>
WSVD_DEV void compute_qtilde(const AttnParams& p, const void* bk_lds, const float* q_lds, float* qts /* LDS [G][R] */) {
  const int tid = threadIdx.x;
  const int cpr = p.d >> 3;                 // chunks per row: 16 (d = 128) or 8 (d = 64)
  const int n_chunks = R * cpr;
  const int nt = blockDim.x;
  for (int ch = tid; ch < (n_chunks + nt - 1) / nt * nt; ch += nt) {   // uniform trip count: DPP needs whole rows active
    const bool on = ch < n_chunks;
    const int j = on ? ch / cpr : 0, cb = on ? ch % cpr : 0;
    float bk[8];
    lds_load8<ESZ>(bk_lds, j * p.d + cb * 8, bk);
    for (int g = 0; g < p.G; g++) {
      const v4f q0 = *(const v4f*)(q_lds + g * p.d + cb * 8), q1 = *(const v4f*)(q_lds + g * p.d + cb * 8 + 4);
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 4; i++) { acc = fmaf(bk[i], q0[i], acc); acc = fmaf(bk[4 + i], q1[i], acc); }
      acc = cpr == 16 ? group_sum<16>(acc) : group_sum<8>(acc);
      if (on && cb == 0) qts[g * R + j] = acc * p.c_scale;
    }
  }
  __syncthreads();
}

// Tail of every attention kernel.  On entry Msh[g], Lsh[g], Ush[g*R+j] hold this workgroup's running
// max (log2 domain), sum and un-normalised latent-space accumulator, visible to all threads.
// If the sequence was split over several workgroups, the workgroup of the LAST split finishes the sequence and the
// others push their (m, l, u) to it: every value travels as one 8-byte word {value, tag}, written with an agent-scope
// store, so a word is either absent (zero, or whatever an earlier launch left: never the tag) or complete, and the
// finisher needs no ticket and no second trip: it asks for the words and asks again until they carry the tag.  Workgroups
// are dispatched in order of their linear id and the splits of a (sequence, kv head) have increasing ids, so everything
// the finisher waits for belongs to workgroups that were dispatched before it and wait for nothing themselves: the
// wait ends whatever the number of workgroups the chip holds at a time (it is bounded all the same, and reports
// through the status word).  The finisher folds the splits in split order (deterministic) and clears the words, so the
// area is all zeros between launches.
// Returns false in the workgroups that only delivered a partial (they are done); true in the one that now holds the
// whole sequence's (m, l, u) in Msh, Lsh, Ush, visible to all of its threads.
constexpr uint32_t kSplitTag = 0x53504C54u;
WSVD_DEV unsigned long long split_word(float v) { return ((unsigned long long)kSplitTag << 32) | (unsigned long long)__float_as_uint(v); }

template <int R>
WSVD_DEV bool attn_merge_splits(const AttnParams& p, const WorkItem& w, float* Msh, float* Lsh, float* Ush, int* flag_sh) {
  const int tid = threadIdx.x;
  const int G = p.G;
  if (w.n_splits <= 1) return true;
  unsigned long long* const base = p.partials + (((size_t)w.b * p.Hq + (size_t)w.kv * G) * p.n_chunks) * (R + 2);
  const size_t g_stride = (size_t)p.n_chunks * (R + 2);          // words between two heads of the group
  if (w.chunk != w.n_splits - 1) {
    for (int i = tid; i < G * (R + 2); i += blockDim.x) {
      const int g = i / (R + 2), k = i % (R + 2);
      const float v = k == 0 ? Msh[g] : k == 1 ? Lsh[g] : Ush[g * R + (k - 2)];
      __hip_atomic_store(base + g * g_stride + (size_t)w.chunk * (R + 2) + k, split_word(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return false;
  }
  const int n_in = w.n_splits - 1;                               // splits pushed to this workgroup
  constexpr int NI = 4;                                          // passes over the G * R <= 1024 items, >= 256 threads
  float Mres[NI], Lres[NI], Ures[NI];
  bool timed_out = false;
#pragma unroll
  for (int it = 0; it < NI; it++) {
    const int i = tid + it * (int)blockDim.x;
    if (i < G * R) {
      const int g = i / R, jj = i % R;
      const unsigned long long* src = base + g * g_stride;
      float M = -INFINITY, L = 0.f, U = 0.f;
      for (int c0 = 0; c0 < n_in; c0 += 8) {
        unsigned long long wm[8], wl[8], wu[8];
        int budget = 1 << 14;
        for (;;) {
#pragma unroll
          for (int k = 0; k < 8; k++) {
            if (k == 0 || c0 + k < n_in) {                       // workgroup-uniform: only the splits that exist are asked for
              const unsigned long long* pc = src + (size_t)(c0 + k) * (R + 2);
              wm[k] = __hip_atomic_load(pc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              wl[k] = __hip_atomic_load(pc + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              wu[k] = __hip_atomic_load(pc + 2 + jj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
              wm[k] = wm[0]; wl[k] = wl[0]; wu[k] = wu[0];       // a duplicate of slot c0: masked in the fold below
            }
          }
          bool all = true;
#pragma unroll
          for (int k = 0; k < 8; k++)
            all = all && (uint32_t)(wm[k] >> 32) == kSplitTag && (uint32_t)(wl[k] >> 32) == kSplitTag && (uint32_t)(wu[k] >> 32) == kSplitTag;
          if (all) break;
          if (--budget == 0) { timed_out = true; break; }
          __builtin_amdgcn_s_sleep(1);
        }
        float mv[8], lv[8], uv[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
          mv[k] = __uint_as_float((uint32_t)wm[k]); lv[k] = __uint_as_float((uint32_t)wl[k]); uv[k] = __uint_as_float((uint32_t)wu[k]);
        }
        float Mn = M;
#pragma unroll
        for (int k = 0; k < 8; k++) Mn = fmaxf(Mn, mv[k]);                        // a duplicate cannot change a max
        // 0 on the first batch (M = -inf); a slot that saw no row in any split so far keeps M = Mn = -inf
        const float keep = M == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(M - Mn);
        L *= keep; U *= keep;
#pragma unroll
        for (int k = 0; k < 8; k++) {
          const float e = (c0 + k < n_in && mv[k] != -INFINITY) ? __builtin_amdgcn_exp2f(mv[k] - Mn) : 0.f;
          L = fmaf(lv[k], e, L);
          U = fmaf(uv[k], e, U);
        }
        M = Mn;
      }
      // this workgroup's own split comes last
      const float mo = Msh[g];
      const float Mn = fmaxf(M, mo);
      const float keep = M == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(M - Mn);
      const float eo = mo == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mo - Mn);
      Ures[it] = fmaf(Ush[i], eo, U * keep);
      Lres[it] = fmaf(Lsh[g], eo, L * keep);
      Mres[it] = Mn;
    }
  }
  if (timed_out) atomicExch(p.err_word, (int)WSVD_E_HIP);       // never seen; keeps the wait finite
  __syncthreads();                                               // every thread has read the words and the LDS values it needs
#pragma unroll
  for (int it = 0; it < NI; it++) {
    const int i = tid + it * (int)blockDim.x;
    if (i < G * R) {
      const int g = i / R, jj = i % R;
      Ush[i] = Ures[it];
      if (jj == 0) { Lsh[g] = Lres[it]; Msh[g] = Mres[it]; }
      unsigned long long* dst = base + g * g_stride;
      for (int c = 0; c < n_in; c++) {
        __hip_atomic_store(dst + (size_t)c * (R + 2) + 2 + jj, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (jj == 0) {
          __hip_atomic_store(dst + (size_t)c * (R + 2), 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(dst + (size_t)c * (R + 2) + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }
  __syncthreads();
  (void)flag_sh;
  return true;
}

template <int R, int ESZ>
WSVD_DEV void attn_tail(const AttnParams& p, const WorkItem& w, float* Msh, float* Lsh, float* Ush, int* flag_sh,
                        const void* bv_lds) {
  const int tid = threadIdx.x;
  const int G = p.G;
  if (!attn_merge_splits<R>(p, w, Msh, Lsh, Ush, flag_sh)) return;
  WSVD_STAMP(p.timeline, ((int)blockIdx.z * (int)gridDim.y + (int)blockIdx.y) * (int)gridDim.x + (int)blockIdx.x, threadIdx.x >> 6, 11);
  if (!bv_lds) {
    // latent-output variant: the normalised accumulator itself (B_V lives in the output projection)
    for (int i = tid; i < G * R; i += blockDim.x)
      p.out[((size_t)w.b * p.Hq + first_head(p, w.kv)) * R + i] = Ush[i] / Lsh[i / R];
    return;
  }
  // out[b, h, c] = sum_j (U[g][j] / L[g]) * B_V[kv][j][c], B_V[kv] staged in LDS.
  // Four adjacent lanes share an output (a quarter of the latent dims each) and add up through DPP, which keeps
  // the dependent LDS-read chain short at the very end of the kernel.
  if (ESZ == 2) {
    // bf16 factors: two adjacent columns per lane (one LDS dword carries both), so half as many passes
    const int half_d = p.d >> 1, n_pair = G * half_d;
    const uint32_t* bv32 = (const uint32_t*)bv_lds;
    for (int i0 = 0; i0 < n_pair * 4; i0 += blockDim.x) {   // uniform trip count: whole quads stay active
      const int i = i0 + tid;
      const int o = min(i >> 2, n_pair - 1), part = i & 3;
      const int g = o / half_d, c2 = o % half_d;
      float a0 = 0.f, a1 = 0.f;
#pragma unroll
      for (int jj = 0; jj < R / 4; jj++) {
        const int j = part * (R / 4) + jj;
        const uint32_t bb = bv32[j * half_d + c2];
        const float u = Ush[g * R + j];
        a0 = fmaf(u, __uint_as_float(bb << 16), a0);
        a1 = fmaf(u, __uint_as_float(bb & 0xFFFF0000u), a1);
      }
      a0 = group_sum<4>(a0);
      a1 = group_sum<4>(a1);
      if (part == 0 && (i >> 2) < n_pair) {
        const float L = Lsh[g];
        out_put2(p, ((size_t)w.b * p.Hq + first_head(p, w.kv) + g) * p.d + 2 * c2, L > 0.f ? a0 / L : 0.f,
                 L > 0.f ? a1 / L : 0.f);                                          // no visible row at all: zeros
      }
    }
    return;
  }
  const int n_out = G * p.d;
  for (int i0 = 0; i0 < n_out * 4; i0 += blockDim.x) {     // uniform trip count: whole quads stay active
    const int i = i0 + tid;
    const int o = min(i >> 2, n_out - 1), part = i & 3;
    const int g = o / p.d, c = o % p.d;
    float acc = 0.f;
#pragma unroll
    for (int jj = 0; jj < R / 4; jj++) {
      const int j = part * (R / 4) + jj;
      acc = fmaf(Ush[g * R + j], ((const float*)bv_lds)[j * p.d + c], acc);
    }
    acc = group_sum<4>(acc);
    if (part == 0 && (i >> 2) < n_out) out_put(p, ((size_t)w.b * p.Hq + first_head(p, w.kv) + g) * p.d + c, acc / Lsh[g]);
  }
}
