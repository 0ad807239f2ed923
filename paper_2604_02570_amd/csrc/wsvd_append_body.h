// Device-side pieces of the latent append shared by the stand-alone append kernels and the fused decode-step
// kernel: parameters, the row quantise-and-store routines, the slice hand-off and the matrix-core projection.
#pragma once
#include "wsvd_dev.h"
#include "wsvd_internal.h"

struct AppendParams {
  const void* x;             // [B,E]
  const uint16_t* x_scale;   // fp16 [B] iff x_dtype == I8
  const void* A[2];          // A_K, A_V packed (a_packed_offset)
  uint8_t* codes[2];
  uint16_t* meta[2];
  int* seq_lens;
  float* partials;           // [2][Hkv][ES][B][R]
  int* tickets;              // [2*Hkv] per (plane, kv head) tickets, then [1] the readers' ticket
  int* err_word;
  int B, E, Hkv, t_cap, ES, ESL;
  int x_dtype, factor_dtype, latent_dtype;
  // fused decode step: rows are stored with write-through (agent-scope) stores and announced through flags[plane*Hkv+kv]
  // = epoch instead of the length update, which the step kernel does once every workgroup has finished
  int fused;
  int epoch;
  int* flags;
  // prefill of one sequence: all B rows of x are consecutive tokens of sequence one_seq (>= 0); token i goes to row
  // seq_lens[one_seq] + i and the length advances by B.  -1: one token per sequence (decode).
  int one_seq;
  long long* timeline;       // profiling build: stamp buffer (see WSVD_STAMP), else null
  // paged cache only (else null): codes / meta are pools of n_pages pages, a page = page_rows rows of every kv head
  const int* block_table;    // [B][max_pages]
  int page_rows, max_pages, n_pages;
  // projection-only launch of the decode step (k_append_split<.., true>): partial sums [slice][plane][B][Hkv * R] fp32,
  // and one word per sequence saying that its length was advanced and the row is still to be written
  float* defer_out;
  int* pending;
};

// which sequence a row of x belongs to, and the cache row it goes to given that sequence's length
WSVD_DEV int append_seq_of(const AppendParams& p, int b) { return p.one_seq >= 0 ? p.one_seq : b; }
WSVD_DEV int append_target_row(const AppendParams& p, int b) {
  const int n = p.seq_lens[append_seq_of(p, b)];
  return (p.one_seq >= 0 && n >= 0) ? n + b : n;
}

// Row stores.  In the fused decode step the attention workgroups of the SAME launch read the new row, possibly from
// another XCD, so there the bytes go out with agent-scope stores.
WSVD_DEV void put_u8(const AppendParams& p, uint8_t* a, uint8_t v) {
  if (p.fused) __hip_atomic_store(a, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); else *a = v;
}
WSVD_DEV void put_u16(const AppendParams& p, uint16_t* a, uint16_t v) {
  if (p.fused) __hip_atomic_store(a, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); else *a = v;
}
// after a workgroup's row stores: all of them acknowledged, then the flag
WSVD_DEV void append_announce(const AppendParams& p, int pl, int kv) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // row bytes at the device's coherence point, stores drained
  wait_vmem_done();
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_store(p.flags + pl * p.Hkv + kv, p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kAppendBB = 8;       // batch rows per pass
constexpr int kAppendMaxESL = 256; // d_model slice per workgroup (vector-ALU kernel)
constexpr int kAppendMaxB = 1024;  // sequences per call
constexpr int kAppendMfmaESL = 512; // largest d_model slice of the MFMA kernel (its hidden-state staging in LDS)

WSVD_DEV float load_x(const AppendParams& p, int b, int e) {
  const size_t idx = (size_t)b * p.E + e;
  if (p.x_dtype == WSVD_I8) return (float)((const int8_t*)p.x)[idx] * f16_bits_to_f32(p.x_scale[b]);
  return load_as_f32(p.x, idx, p.x_dtype);
}

// Where row t of (b, kv) lives: the plane of its codes (row_bytes per row), the index of its metadata entry, and the row
// index inside that plane.  Contiguous cache: one plane of t_cap rows per (b, kv).  Paged cache (quantised latents): the
// page block_table[b][t / page_rows] of the pools holds page_rows rows of every kv head in the same layout; an entry
// outside the pools reports WSVD_E_SHAPE and the row goes to page 0's slot of nobody (ok = false: not stored).
struct RowAddr {
  uint8_t* plane;
  size_t meta;
  int t;
  bool ok;
};
WSVD_DEV RowAddr append_row_addr(const AppendParams& p, int pl, int b, int kv, int t, int row_bytes) {
  RowAddr a;
  if (!p.block_table) {
    const size_t ph = (size_t)b * p.Hkv + kv;
    a.plane = p.codes[pl] + ph * (size_t)p.t_cap * row_bytes; a.meta = ph * p.t_cap + t; a.t = t; a.ok = true;
    return a;
  }
  const int pg = min(t / p.page_rows, p.max_pages - 1);
  int phys = p.block_table[(size_t)b * p.max_pages + pg];
  a.ok = phys >= 0 && phys < p.n_pages;
  if (!a.ok) { phys = 0; atomicExch(p.err_word, (int)WSVD_E_SHAPE); }
  const size_t slot = (size_t)phys * p.Hkv + kv;
  a.t = t - pg * p.page_rows;
  a.plane = p.codes[pl] + slot * (size_t)p.page_rows * row_bytes; a.meta = slot * p.page_rows + a.t;
  return a;
}

// Store one latent row with R cooperating lanes (a half wave for R = 32, a wave for R = 64, 16 lanes for R = 16):
// lane j holds c_j.  Same arithmetic per element as quantize_row_i8 / quantize_row_i4 (max / min are exact in any
// order), so the stored bits are identical to those routines'.
template <int R>
WSVD_DEV float lanes_max(float x) {   // max over the R adjacent lanes that hold one row
  x = row16_max(x);
  if (R == 16) return x;
  const int lane = threadIdx.x & 63;
  const float a = fmaxf(lane_bcast(x, 0), lane_bcast(x, 16)), b = fmaxf(lane_bcast(x, 32), lane_bcast(x, 48));
  return R == 64 ? fmaxf(a, b) : (lane < 32 ? a : b);
}

// `on` (the same for all lanes of a row): false = take part in the reductions, form no address, store nothing.
template <int R>
WSVD_DEV void store_row_lanes(const AppendParams& p, int pl, int b, int kv, int t, int j, float c, bool on = true) {
  const size_t ph = (size_t)b * p.Hkv + kv;
  if (p.latent_dtype == WSVD_F32) {
    ((float*)p.codes[pl])[(ph * p.t_cap + t) * R + j] = c;
  } else if (p.latent_dtype == WSVD_BF16) {
    ((uint16_t*)p.codes[pl])[(ph * p.t_cap + t) * R + j] = f32_to_bf16_rne(c);
  } else if (p.latent_dtype == WSVD_I8) {
    const float a = lanes_max<R>(fabsf(c));
    uint16_t sh = 0x3C00u;
    if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
    const float sc = f16_bits_to_f32(sh);
    const float v = fminf(fmaxf(__builtin_rintf(c / sc), -127.f), 127.f);
    RowAddr ra;
    ra.ok = false;
    if (on) ra = append_row_addr(p, pl, b, kv, t, R);
    if (ra.ok) {
      put_u8(p, ra.plane + (pl == 0 ? i8_k_offset(ra.t, j, R) : i8_v_offset(ra.t, j, R)), (uint8_t)(int8_t)(int)v);
      if (j == 0) put_u16(p, &p.meta[pl][ra.meta], sh);
    }
  } else {  // I4, R == 32
    const float hi = lanes_max<R>(fmaxf(c, 0.f)), lo = -lanes_max<R>(fmaxf(-c, 0.f));
    uint16_t sh = 0x3C00u;
    float z = 0.f;
    const bool flat = (hi == lo);
    if (!flat) sh = guard_scale_f16((hi - lo) / 15.0f);
    const float sc = f16_bits_to_f32(sh);
    if (!flat) z = fminf(fmaxf(__builtin_rintf(-lo / sc), 0.f), 15.f);
    const int zi = (int)z;
    int q = (int)fminf(fmaxf(__builtin_rintf(c / sc), -64.f), 64.f) + zi;
    q = q < 0 ? 0 : (q > 15 ? 15 : q);
    RowAddr ra;
    ra.ok = false; ra.plane = nullptr; ra.t = 0; ra.meta = 0;
    if (on) ra = append_row_addr(p, pl, b, kv, t, R / 2);
    uint8_t* plane = ra.plane;
    int nib;
    if (pl == 0) {
      // dims (j, j+1) share a byte: the odd lane hands its code to the even lane
      const int qn = __builtin_amdgcn_update_dpp(0, q, kDppQuadSwap1, 0xF, 0xF, true);
      if ((j & 1) == 0 && ra.ok) put_u8(p, plane + i4_k_offset(ra.t, j, &nib), (uint8_t)(q | (qn << 4)));
    } else if (ra.ok) {
      // tokens (t, t^1) share each byte; the other token was (or will be) written by a different launch
      uint8_t* bp = plane + i4_v_offset(ra.t, j, &nib);
      const uint8_t old = *bp;
      put_u8(p, bp, nib ? (uint8_t)((old & 0x0F) | (q << 4)) : (uint8_t)((old & 0xF0) | q));
    }
    if (j == 0 && ra.ok) {
      put_u16(p, &p.meta[pl][ra.meta * 2], sh);
      put_u16(p, &p.meta[pl][ra.meta * 2 + 1], f32_to_f16_bits_rne((float)zi));
    }
  }
}

// Bookkeeping shared by both append kernels.
template <int R>
WSVD_DEV void append_store_rows(const AppendParams& p, int pl, int kv, int b0, int nb, float (*crow)[R + 1], const int* n_sh) {
  // R lanes per row; rows_per_pass = blockDim / R rows at a time (whole waves stay converged for the lane reductions)
  const int j = threadIdx.x % R, rsub = threadIdx.x / R, rpp = blockDim.x / R;
  for (int r0 = 0; r0 < nb; r0 += rpp) {
    const int row = min(r0 + rsub, nb - 1);            // clamped: surplus lanes redo the last row, then skip the store
    const int n = n_sh[b0 + row];
    const bool on = (r0 + rsub < nb) && n >= 0 && n < p.t_cap;
    const float c = crow[row][j];
    if (p.latent_dtype == WSVD_I8 || p.latent_dtype == WSVD_I4) {
      // the reductions need every lane of the wave: the lanes of a row that must not be stored (the surplus ones of a
      // ragged tail, a sequence at capacity) go through them on the clamped row's values and skip the stores.  (A
      // single sequence, or the odd row of a group, used to fall back to one lane quantising the row by itself:
      // 2 us more for the launch.)
      if (__builtin_amdgcn_ballot_w64(on) != 0ull) store_row_lanes<R>(p, pl, append_seq_of(p, b0 + row), kv, n, j, c, on);
    } else if (on) {
      store_row_lanes<R>(p, pl, append_seq_of(p, b0 + row), kv, n, j, c);
    }
  }
}

// sequence lengths -> LDS
WSVD_DEV void append_read_lens(const AppendParams& p, int* n_sh) {
  for (int b = threadIdx.x; b < p.B; b += blockDim.x) n_sh[b] = append_target_row(p, b);
  __syncthreads();
}

// Advancing the sequence lengths only has to wait until every workgroup that USES the old ones (the 2*Hkv that end
// up storing the rows of a plane and kv head) holds its copy; the consumer of the new lengths is a later kernel.
// So such a workgroup draws a ticket as soon as it knows its role, before it sums and stores, and looks at the
// answer on its way out: the atomic's round trip overlaps the remaining work.  Whoever drew the last ticket
// advances the lengths (or reports a full sequence).
WSVD_DEV int append_reader_ticket(const AppendParams& p) {
  return __hip_atomic_fetch_add(p.tickets + 2 * p.Hkv, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
WSVD_DEV void append_bump(const AppendParams& p, const int* n_sh, int ticket /* thread 0's draw */, int* flag_sh) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const int last = (ticket == 2 * p.Hkv - 1);
    if (last) __hip_atomic_store(p.tickets + 2 * p.Hkv, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag_sh = last;
  }
  __syncthreads();
  if (!*flag_sh) return;
  if (p.one_seq >= 0) {
    // the rows that fitted were stored; a prompt that does not fit leaves the sequence full and is reported
    if (threadIdx.x == 0) {
      const int n0 = n_sh[0];
      if (n0 >= 0) p.seq_lens[p.one_seq] = min(n0 + p.B, p.t_cap);
      if (n0 < 0 || n0 + p.B > p.t_cap) atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
    }
    return;
  }
  for (int b = threadIdx.x; b < p.B; b += blockDim.x) {
    const int n = n_sh[b];
    if (n >= 0 && n < p.t_cap) p.seq_lens[b] = n + 1;
    else atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
  }
}

// Several d_model slices: hand this workgroup's partials over and let the last arriver of the (plane, kv head)
// continue.  Returns false for every other workgroup.  On return crow holds nothing yet; the caller sums slices.
WSVD_DEV bool append_slice_ticket(const AppendParams& p, int pl, int kv, int* flag_sh) {
  wait_vmem_done();  // this thread's partial stores are acknowledged ...
  __syncthreads();   // ... and so are everybody's, before the ticket is taken
  if (threadIdx.x == 0) {
    int* t = p.tickets + pl * p.Hkv + kv;
    const int old = __hip_atomic_fetch_add(t, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == p.ES - 1);
    if (last) __hip_atomic_store(t, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag_sh = last;
  }
  __syncthreads();
  return *flag_sh != 0;
}

template <int R>
WSVD_DEV void append_finish(const AppendParams& p, int pl, int kv, float (*crow)[R + 1], int* flag_sh, const int* n_sh) {
  const int tid = threadIdx.x;
  if (append_slice_ticket(p, pl, kv, flag_sh)) {
    const int ticket = (tid == 0 && !p.fused) ? append_reader_ticket(p) : 0;   // n_sh is complete in every workgroup by now
    const float* pbase = p.partials + (((size_t)pl * p.Hkv + kv) * p.ES) * p.B * R;
    for (int b0 = 0; b0 < p.B; b0 += 64) {
      const int nb = min(64, p.B - b0);
      __syncthreads();
      // Slices are summed in order.  The loads bypass the caches and cost a full round trip each, so every thread
      // requests its (up to) four elements x 8 slices together (index clamped, surplus masked) instead of one
      // element per trip.
      for (int i0 = 0; i0 < nb * R; i0 += 4 * (int)blockDim.x) {
        float sum[4] = {0.f, 0.f, 0.f, 0.f};
        for (int k0 = 0; k0 < p.ES; k0 += 8) {
          float v[4][8];
#pragma unroll
          for (int it = 0; it < 4; it++) {
            const int i = min(i0 + it * (int)blockDim.x + tid, nb * R - 1);
#pragma unroll
            for (int k = 0; k < 8; k++) v[it][k] = agent_load(pbase + ((size_t)min(k0 + k, p.ES - 1) * p.B + b0) * R + i);
          }
#pragma unroll
          for (int it = 0; it < 4; it++)
#pragma unroll
            for (int k = 0; k < 8; k++) sum[it] += (k0 + k < p.ES) ? v[it][k] : 0.f;
        }
#pragma unroll
        for (int it = 0; it < 4; it++) {
          const int i = i0 + it * (int)blockDim.x + tid;
          if (i < nb * R) crow[i / R][i % R] = sum[it];
        }
      }
      __syncthreads();
      append_store_rows<R>(p, pl, kv, b0, nb, crow, n_sh);
    }
    if (p.fused) append_announce(p, pl, kv);
    else append_bump(p, n_sh, ticket, flag_sh);
  }
}

// blockIdx.x -> (d_model slice s, kv head, plane)
WSVD_DEV void append_coords(const AppendParams& p, int id, int& s, int& kv, int& pl) {
  s = id % p.ES; id /= p.ES;
  kv = id % p.Hkv;
  pl = id / p.Hkv;
}

// ---------------------------------------------------------------- MFMA path (bf16 factors, bf16 x)
// D[latent channel][sequence] += A^T tile (rows = channels, k = 16 consecutive e) x X^T tile (columns = sequences).
// Operand layout (checked on hardware): lane L holds row / column L%32 and k = 8*(L/32)..+7, i.e. 16 contiguous bytes
// of a factor row or of a hidden-state row.  Each of the 4 waves takes a quarter of the workgroup's d_model slice.
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// NT = launch bound.  The workgroup's d_model slice [e0, e0 + ESL) is divided over its NW = blockDim/64 waves; a wave
// walks its part in chunks of 4 k-steps (64 elements), the next chunk's operands in flight while the current one
// multiplies.  With ES == 1 (one workgroup per plane and kv head, up to 16 waves) there is no cross-workgroup
// hand-off at all.  Sequence lengths are requested first and land in LDS together with the hidden states.
// NG = groups of 32 sequences that share one pass over the factors (1, or 2 for batches above 32: the factor operand
// is loaded once and multiplied with both groups' hidden states)
template <int R, int NG>
struct AppendMfmaShared {
  static constexpr int RW = R <= 32 ? 8 : 4;   // waves reduced per LDS round
  float crow[64][R + 1];
  int flag_sh;
  int n_sh[kAppendMaxB];
  // The hidden-state slice and the cross-wave reduction buffer are never live together (a barrier separates the
  // last operand read from the first partial written, and the last sum from the next slice), so they share storage.
  union {
    // hidden-state slice of up to 32 * NG sequences, row stride = 4 dwords mod 32 banks so that the 16-byte operand
    // reads of 8 consecutive sequences cover all banks once
    __attribute__((aligned(16))) uint16_t xs[32 * NG][kAppendMfmaESL + 8];
    float red[RW][32][R + 1];                  // [wave in round][sequence in group][channel]
  };
};

// wg = index of the workgroup among the append workgroups of the launch
template <int R, int NG>
WSVD_DEV void append_mfma_body(const AppendParams& p, AppendMfmaShared<R, NG>& sh, int wg) {
  constexpr int RT = R / 32;                  // 32-channel row tiles (R = 16 uses half a tile)
  constexpr int RTC = RT > 0 ? RT : 1;
  constexpr int KS = 4;                       // k-steps of 16 per chunk
  constexpr int RW = AppendMfmaShared<R, NG>::RW;
  constexpr int NLEN = kAppendMaxB / 256;     // sequence lengths per thread (blockDim >= 256)
  auto& red = sh.red;
  auto& crow = sh.crow;
  int& flag_sh = sh.flag_sh;
  auto& n_sh = sh.n_sh;
  auto& xs = sh.xs;

  int s, kv, pl;
  append_coords(p, wg, s, kv, pl);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NW = blockDim.x >> 6;
  int nreg[NLEN];
#pragma unroll
  for (int i = 0; i < NLEN; i++) nreg[i] = append_target_row(p, min(i * (int)blockDim.x + tid, p.B - 1));

  const int ew = p.ESL / NW;                                 // d_model elements per wave (multiple of 16)
  const int ks_n = ew / 16;
  const int e_w = s * p.ESL + wave * ew;
  const int col = lane & 31, g = lane >> 5;
  float* part = p.partials + ((((size_t)pl * p.Hkv + kv) * p.ES + s) * p.B) * R;
  const uint16_t* Ap = (const uint16_t*)p.A[pl];
  const uint16_t* xp = (const uint16_t*)p.x;
  bool lens_done = false;
  int ticket = 0;

  for (int b0 = 0; b0 < p.B; b0 += 32 * NG) {
    const int nb = min(32 * NG, p.B - b0);
    int xrow[NG];
    v16f acc[NG][RTC];
#pragma unroll
    for (int gi = 0; gi < NG; gi++) {
      xrow[gi] = min(32 * gi + col, nb - 1);
#pragma unroll
      for (int rt = 0; rt < RTC; rt++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[gi][rt][v] = 0.f;
    }
    // factor operands of one chunk: unconditional loads (k-step clamped to the wave's last one); the hidden-state
    // operands come from the LDS copy, which the whole workgroup fills with coalesced 16-byte loads
    v8bf aop[2][RTC][KS];
    auto load_chunk = [&](int buf, int c0) {
#pragma unroll
      for (int k = 0; k < KS; k++) {
        const int kk = min(c0 + k, ks_n - 1);
#pragma unroll
        for (int rt = 0; rt < RTC; rt++)
          aop[buf][rt][k] = *(const v8bf*)(Ap + (((size_t)(kv * RTC + rt) * (size_t)(p.E >> 4) + (size_t)((e_w >> 4) + kk)) * 64 + lane) * 8);
      }
    };
    auto mul_chunk = [&](int buf, int c0) {
#pragma unroll
      for (int k = 0; k < KS; k++)
        if (c0 + k < ks_n) {
#pragma unroll
          for (int gi = 0; gi < NG; gi++) {
            const v8bf xo = *(const v8bf*)&xs[xrow[gi]][wave * ew + (c0 + k) * 16 + g * 8];
#pragma unroll
            for (int rt = 0; rt < RTC; rt++)
              acc[gi][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[buf][rt][k], xo, acc[gi][rt], 0, 0, 0);
          }
        }
    };
    load_chunk(0, 0);
    {
      const int ppr = p.ESL >> 3;                       // 16-byte pieces per row
      __syncthreads();                                  // the previous group's operand reads are done
      // four pieces per thread and trip, all four loads in flight before the first LDS write (one piece per trip
      // made every trip a memory round trip of its own)
      for (int i0 = 0; i0 < nb * ppr; i0 += 4 * (int)blockDim.x) {
        v4i piece[4];
#pragma unroll
        for (int it = 0; it < 4; it++) {
          const int i = min(i0 + it * (int)blockDim.x + tid, nb * ppr - 1);
          piece[it] = *(const v4i*)(xp + (size_t)(b0 + i / ppr) * p.E + s * p.ESL + (i % ppr) * 8);
        }
#pragma unroll
        for (int it = 0; it < 4; it++) {
          const int i = i0 + it * (int)blockDim.x + tid;
          if (i < nb * ppr) *(v4i*)&xs[i / ppr][(i % ppr) * 8] = piece[it];
        }
      }
      if (!lens_done) {
        // the lengths were requested before everything else, so they are here by now
#pragma unroll
        for (int i = 0; i < NLEN; i++) {
          const int b = i * (int)blockDim.x + tid;
          if (b < p.B) n_sh[b] = nreg[i];
        }
      }
      __syncthreads();
      if (!lens_done && tid == 0 && p.ES == 1 && !p.fused) ticket = append_reader_ticket(p);   // the lengths are complete in LDS
      lens_done = true;
    }
    for (int c0 = 0; c0 < ks_n; c0 += 2 * KS) {
      load_chunk(1, c0 + KS);
      mul_chunk(0, c0);
      load_chunk(0, c0 + 2 * KS);
      mul_chunk(1, c0 + KS);
    }
    // cross-wave sum in a fixed order: per group of 32 sequences, rounds of RW waves through LDS
#pragma unroll
    for (int gi = 0; gi < NG; gi++) {
      const int nbg = min(32, nb - 32 * gi);             // sequences of this group (<= 0: none)
      if (nbg <= 0) break;
      for (int r0 = 0; r0 < NW; r0 += RW) {
        __syncthreads();
        if (wave >= r0 && wave < r0 + RW) {
#pragma unroll
          for (int rt = 0; rt < RTC; rt++)
#pragma unroll
            for (int v = 0; v < 16; v++) {
              // lane holds sequence column `col`, channel rows 8*(v/4) + 4*g + v%4
              const int ch = rt * 32 + 8 * (v / 4) + 4 * g + (v % 4);
              if (ch < R) red[wave - r0][col][ch] = acc[gi][rt][v];
            }
        }
        __syncthreads();
        const int nr = min(RW, NW - r0);
        for (int i = tid; i < nbg * R; i += blockDim.x) {
          const int bb = i / R, jj = i % R;
          float sum = r0 == 0 ? 0.f : crow[32 * gi + bb][jj];
          for (int k = 0; k < nr; k++) sum += red[k][bb][jj];
          crow[32 * gi + bb][jj] = sum;
        }
      }
    }
    __syncthreads();
    if (p.ES == 1) {
      append_store_rows<R>(p, pl, kv, b0, nb, crow, n_sh);
    } else {
      for (int i = tid; i < nb * R; i += blockDim.x) agent_store(&part[(size_t)(b0 + i / R) * R + i % R], crow[i / R][i % R]);
    }
  }
  if (p.ES != 1) append_finish<R>(p, pl, kv, crow, &flag_sh, n_sh);
  else if (p.fused) append_announce(p, pl, kv);
  else append_bump(p, n_sh, ticket, &flag_sh);
}

template <int R, int NT, int NG>
__global__ __launch_bounds__(NT) void k_append_mfma(AppendParams p) {
  __shared__ AppendMfmaShared<R, NG> sh;
  append_mfma_body<R, NG>(p, sh, blockIdx.x);
}

