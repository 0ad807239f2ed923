// Causal attention of a block of query tokens over the int8 latent cache, tiled for the matrix cores (the attention
// of prefilling, Section 3.4, in latent space).
//
// With no rotation between the reconstruction and the product, q K^T = (q B_K^T) C_K^T and P V = (P C_V) B_V: the
// whole score / softmax / value loop runs on latents of dimension r instead of keys and values of dimension d.
//   prologue  Q~^T [r x 32 queries] = B_K q^T                       bf16 MFMA, operands straight from global memory
//   loop      S^T [32 keys x 32 queries] = C_K Q~^T                 fp16 MFMA: codes are exact in fp16, Q~ is an fp16 pair
//             online softmax down the columns (a lane owns one query column: running max and sum are per lane)
//             U^T [r x 32 queries] += (diag(s_V) C_V)^T P           fp16 MFMA: code * scale and P rounded to fp16 (2^-12
//                                                                   relative each), P through LDS
//   epilogue  O^T [d x 32 queries] = B_V^T (U / l)                  bf16 MFMA, U an bf16 pair
// The loop is bound by the vector ALU (the products are a few per cent of its time), so it is written to spend few
// vector instructions per score: byte-permute code conversion, no masks on blocks every query sees whole, the
// accumulator rescaled only when some running maximum moved, single-term fp16 operands for the value product.
// One wavefront per (sequence, kv head, block of 32 query rows); a query row is a (token, head) pair, token-major, so
// the G heads that share a kv head share the stream too.  The cache blocks are read in the layout the decode kernels
// use (a 32-token block of the K plane is a ready-made operand with row = token, one of the V plane with row = dim).
// 32x32 accumulator layout throughout: lane L holds column L % 32, rows 8 (v / 4) + 4 (L / 32) + v % 4, v = 0..15.
#include <type_traits>
#include "wsvd_dev.h"
#include "wsvd_internal.h"

namespace {

struct PrefillParams {
  const uint16_t* q;          // bf16 [B, Hkv, NR, d], NR = nq * G query rows per kv head (row = token * G + head)
  const uint16_t* BK;         // bf16 [Hkv, R, d]
  const uint16_t* BV;
  const uint8_t* k_codes;
  const uint8_t* v_codes;
  const uint16_t* k_meta;
  const uint16_t* v_meta;
  const int* seq_lens;
  float* out;                 // fp32 [B, Hkv, NR, d]
  int B, Hkv, G, d, t_cap, nq, n_after, NR;
  float c_scale;              // sm_scale * log2(e)
  // paged cache only (else null): the planes are pools of n_pages pages, a page = page_rows rows of every kv head in the
  // layout of a contiguous plane; block_table [B][max_pages]
  const int* block_table;
  int page_rows, max_pages, n_pages;
};

// x as an fp16 pair hi + lo; the fp32 value is pinned in a register so that hi is formed once (a fused
// multiply-convert would otherwise round it a second way for the subtraction)
WSVD_DEV void split_f16(float x, _Float16& hi, _Float16& lo) {
  asm volatile("" : "+v"(x));
  hi = (_Float16)x;
  lo = (_Float16)(x - (float)hi);
}
// x as a bf16 pair (truncation: hi + lo reproduces x to 2^-16 relative)
WSVD_DEV void split_bf16(float x, uint32_t& hi, uint32_t& lo) {
  hi = __float_as_uint(x) & 0xFFFF0000u;
  lo = __float_as_uint(x - __uint_as_float(hi)) & 0xFFFF0000u;
}

template <int R>
__global__ __launch_bounds__(64) void k_prefill_attn(PrefillParams p) {
  constexpr int KK = R / 32;
  __shared__ __attribute__((aligned(16))) float sc_lds[32];             // K scales of the block's 32 tokens
  __shared__ __attribute__((aligned(16))) _Float16 pt[32][40];          // P in fp16, [query][key], padded rows

  const int lane = threadIdx.x, n = lane & 31, g2 = lane >> 5;
  // the last query blocks see the most keys: they are started first, so that the launch does not end on its longest waves
  const int kv = blockIdx.x, qb = gridDim.y - 1 - blockIdx.y, b = blockIdx.z;
  const int nb = p.seq_lens[b];
  const int n_eff = min(max(nb - p.n_after, 0), p.t_cap);
  const int rho = qb * 32 + n;                                          // this lane's query row
  const bool row_ok = rho < p.NR;
  const int rho_c = min(rho, p.NR - 1);
  const int lim = row_ok ? n_eff - p.nq + rho_c / p.G + 1 : 0;          // this query sees keys [0, lim); may be <= 0
  const int rho_last = min(qb * 32 + 31, p.NR - 1);
  const int lim_max = n_eff - p.nq + rho_last / p.G + 1;                // rows are token-major: the last row sees most
  const int n_kblocks = lim_max > 0 ? (lim_max + 31) >> 5 : 0;
  const size_t ph = (size_t)b * p.Hkv + kv;
  float* orow = p.out + (ph * p.NR + rho_c) * p.d;
  if (n_kblocks == 0) {                                                 // nothing visible to any row of the block
    if (row_ok) for (int c = g2 * (p.d >> 1); c < (g2 + 1) * (p.d >> 1); c++) orow[c] = 0.f;
    return;
  }

  // ---- Q~^T = B_K q^T.  Row i of the A operand carries latent dim pi(i) = 16 ((i >> 2) & 1) + 4 (i >> 3) + (i & 3) of
  // its 32-dim block, so that accumulator register v of lane half g2 is dim 16 g2 + v: the order the K blocks use.
  v16f qt[KK];
#pragma unroll
  for (int kk = 0; kk < KK; kk++)
#pragma unroll
    for (int v = 0; v < 16; v++) qt[kk][v] = 0.f;
  {
    const uint16_t* qrow = p.q + (ph * p.NR + rho_c) * p.d + 8 * g2;
    const int dimj = 16 * ((n >> 2) & 1) + 4 * (n >> 3) + (n & 3);
    for (int ks = 0; ks < (p.d >> 4); ks++) {
      const v8bf16 bq = *(const v8bf16*)(qrow + 16 * ks);
#pragma unroll
      for (int kk = 0; kk < KK; kk++) {
        const v8bf16 a = *(const v8bf16*)(p.BK + ((size_t)kv * R + 32 * kk + dimj) * p.d + 16 * ks + 8 * g2);
        qt[kk] = mfma_bf16(a, bq, qt[kk]);
      }
    }
  }
  v8f16 qh[2 * KK], ql[2 * KK];                                         // 16-dim steps of the score contraction
#pragma unroll
  for (int kk = 0; kk < KK; kk++)
#pragma unroll
    for (int v = 0; v < 16; v++) {
      _Float16 h, l;
      split_f16(qt[kk][v] * p.c_scale, h, l);
      qh[2 * kk + (v >> 3)][v & 7] = h;
      ql[2 * kk + (v >> 3)][v & 7] = l;
    }

  const uint8_t* kplane = p.k_codes + ph * (size_t)p.t_cap * R;
  const uint8_t* vplane = p.v_codes + ph * (size_t)p.t_cap * R;
  const uint16_t* kmeta = p.k_meta + ph * (size_t)p.t_cap;
  const uint16_t* vmeta = p.v_meta + ph * (size_t)p.t_cap;

  float m_run = -INFINITY, l_run = 0.f;                                 // l_run: this lane's share of its column's sum
  v16f U[KK];
#pragma unroll
  for (int kk = 0; kk < KK; kk++)
#pragma unroll
    for (int v = 0; v < 16; v++) U[kk][v] = 0.f;

  // one block ahead in registers: codes of both planes, the lane's K scale, the V scales of the lane half's 16 tokens
  v4i kc[KK], vc[KK], vs16[2];
  uint16_t ks_raw;
  // paged cache: the table entries of the first 64 pages, one per lane, fetched once; a block's page is then a lane
  // read with a wave-uniform index (a 32-token block never straddles pages).  Entries outside the pools read page 0
  // (blocks past a sequence's end are never consumed; a bad entry under live rows is the append's to report).
  int page_entry = 0;
  if (p.block_table) page_entry = p.block_table[(size_t)b * p.max_pages + min(lane, p.max_pages - 1)];
  auto load_block = [&](int kb) {
    const uint8_t *kp = kplane, *vp = vplane;
    const uint16_t *km = kmeta, *vm = vmeta;
    if (p.block_table) {
      const int bpp = p.page_rows >> 5;                                 // blocks per page
      const int pg = min(kb / bpp, p.max_pages - 1);
      int e = pg < 64 ? __builtin_amdgcn_readlane(page_entry, __builtin_amdgcn_readfirstlane(pg))
                      : p.block_table[(size_t)b * p.max_pages + pg];
      e = (e >= 0 && e < p.n_pages) ? e : 0;
      const size_t slot = (size_t)e * p.Hkv + kv;
      kp = p.k_codes + slot * (size_t)p.page_rows * R; vp = p.v_codes + slot * (size_t)p.page_rows * R;
      km = p.k_meta + slot * (size_t)p.page_rows; vm = p.v_meta + slot * (size_t)p.page_rows;
      kb -= pg * bpp;
    }
    const size_t off = (size_t)kb * (32 * R) + (size_t)lane * 16;
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      kc[kk] = *(const v4i*)(kp + off + kk * 1024);                     // (plain loads: the other query blocks of this
      vc[kk] = *(const v4i*)(vp + off + kk * 1024);                     //  sequence and head read the same blocks again)
    }
    ks_raw = km[kb * 32 + n];
    vs16[0] = *(const v4i*)(vm + kb * 32 + 16 * g2);
    vs16[1] = *(const v4i*)(vm + kb * 32 + 16 * g2 + 8);
  };
  load_block(0);

  // Blocks below kb_full are seen whole by every query of the wave (and lie inside the written part of the cache): no
  // masks there.  The last one or two blocks take the masked path.
  const int lim_min = n_eff - p.nq + (qb * 32) / p.G + 1;
  const int kb_full = lim_min > 0 ? min(lim_min >> 5, n_kblocks) : 0;

  auto block = [&](int kb, auto masked_c) {
    constexpr bool MASKED = decltype(masked_c)::value;
    // this block's operands out of the load registers, then the next block's loads.  V' = code * s_V in fp16 (the token
    // scales are fp16 already: one packed multiply per two elements).
    v8f16 aK[2 * KK], aV[KK][2];
    v8f16 sv8[2] = {__builtin_bit_cast(v8f16, vs16[0]), __builtin_bit_cast(v8f16, vs16[1])};
    if constexpr (MASKED) {
      // tokens no query of the wave sees (among them rows never written, whose scale may be anything) contribute 0
#pragma unroll
      for (int s = 0; s < 2; s++)
#pragma unroll
        for (int e = 0; e < 8; e++)
          if (kb * 32 + 16 * g2 + 8 * s + e >= lim_max) sv8[s][e] = (_Float16)0;
    }
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      aK[2 * kk] = codes_f16(kc[kk][0], kc[kk][1]);
      aK[2 * kk + 1] = codes_f16(kc[kk][2], kc[kk][3]);
      aV[kk][0] = codes_f16(vc[kk][0], vc[kk][1]) * sv8[0];
      aV[kk][1] = codes_f16(vc[kk][2], vc[kk][3]) * sv8[1];
    }
    sc_lds[n] = f16_bits_to_f32(ks_raw);                                // (both half waves hold the same value)
    load_block(min(kb + 1, n_kblocks - 1));                             // (after the last block: that block again, unused)

    // scores of the block: rows = its 32 tokens, columns = the 32 queries
    const v16f zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    v16f S = mfma_f16(aK[0], qh[0], zero16);                            // (a constant-zero addend: no registers to clear)
    S = mfma_f16(aK[0], ql[0], S);
#pragma unroll
    for (int s = 1; s < 2 * KK; s++) { S = mfma_f16(aK[s], qh[s], S); S = mfma_f16(aK[s], ql[s], S); }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float sc[16];
    float bmax = -INFINITY;
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      const v4f k4 = *(const v4f*)&sc_lds[8 * m4 + 4 * g2];
#pragma unroll
      for (int jj = 0; jj < 4; jj++) {
        const int v = 4 * m4 + jj;
        sc[v] = S[v] * k4[jj];
        if constexpr (MASKED) sc[v] = kb * 32 + 8 * m4 + 4 * g2 + jj < lim ? sc[v] : -INFINITY;
        bmax = fmaxf(bmax, sc[v]);
      }
    }
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32));                           // the other half holds the column's other rows
    const float m_new = fmaxf(m_run, bmax);
    float alpha;
    if constexpr (MASKED) alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
    else alpha = __builtin_amdgcn_exp2f(m_run - m_new);                 // m_new is finite here
    float psum = 0.f;
    float pw[16];
#pragma unroll
    for (int v = 0; v < 16; v++) {
      pw[v] = __builtin_amdgcn_exp2f(sc[v] - m_new);
      if constexpr (MASKED) pw[v] = sc[v] == -INFINITY ? 0.f : pw[v];
      psum += pw[v];
    }
    l_run = fmaf(l_run, alpha, psum);
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {              // the running maxima mostly stand still
#pragma unroll
      for (int kk = 0; kk < KK; kk++)
#pragma unroll
        for (int v = 0; v < 16; v++) U[kk][v] *= alpha;
    }
    // P in fp16 -> LDS, [query][key]: a lane's 16 rows are 4 runs of 4 consecutive keys
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      v4f p4;
#pragma unroll
      for (int jj = 0; jj < 4; jj++) p4[jj] = pw[4 * m4 + jj];
      const v4f16 h4 = __builtin_convertvector(p4, v4f16);
      *(v2i*)&pt[n][8 * m4 + 4 * g2] = __builtin_bit_cast(v2i, h4);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // U^T += V'^T P: rows = latent dims, columns = queries; step s contracts the tokens 16 g2 + 8 s .. + 7 of a half
#pragma unroll
    for (int s = 0; s < 2; s++) {
      const v8f16 bp = *(const v8f16*)&pt[n][16 * g2 + 8 * s];
#pragma unroll
      for (int kk = 0; kk < KK; kk++) U[kk] = mfma_f16(aV[kk][s], bp, U[kk]);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  for (int kb = 0; kb < kb_full; kb++) block(kb, std::false_type{});
  for (int kb = kb_full; kb < n_kblocks; kb++) block(kb, std::true_type{});

  // ---- O^T = B_V^T (U / l).  Register v of U[kk] in lane half g2 is latent dim 32 kk + 8 (v / 4) + 4 g2 + v % 4; the A
  // operand gathers the rows of B_V in that order.
  const float L = l_run + __shfl_xor(l_run, 32);
  const float inv = L > 0.f ? 1.0f / L : 0.f;
  v8bf16 uh[KK][2], ul[KK][2];
#pragma unroll
  for (int kk = 0; kk < KK; kk++)
#pragma unroll
    for (int s = 0; s < 2; s++) {
      v4i hh, ll;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        uint32_t h0, l0, h1, l1;
        split_bf16(U[kk][8 * s + 2 * e] * inv, h0, l0);
        split_bf16(U[kk][8 * s + 2 * e + 1] * inv, h1, l1);
        hh[e] = (int)((h0 >> 16) | h1);
        ll[e] = (int)((l0 >> 16) | l1);
      }
      uh[kk][s] = __builtin_bit_cast(v8bf16, hh);
      ul[kk][s] = __builtin_bit_cast(v8bf16, ll);
    }
  for (int rb = 0; rb < (p.d >> 5); rb++) {
    v16f O;
#pragma unroll
    for (int v = 0; v < 16; v++) O[v] = 0.f;
    const int c = 32 * rb + n;                                          // output channel of this lane's A row
#pragma unroll
    for (int kk = 0; kk < KK; kk++)
#pragma unroll
      for (int s = 0; s < 2; s++) {
        v4i araw;
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const int v0 = 8 * s + 2 * e, v1 = v0 + 1;
          const int j0 = 32 * kk + 8 * (v0 >> 2) + 4 * g2 + (v0 & 3), j1 = 32 * kk + 8 * (v1 >> 2) + 4 * g2 + (v1 & 3);
          const uint32_t e0 = p.BV[((size_t)kv * R + j0) * p.d + c], e1 = p.BV[((size_t)kv * R + j1) * p.d + c];
          araw[e] = (int)(e0 | (e1 << 16));
        }
        const v8bf16 a = __builtin_bit_cast(v8bf16, araw);
        O = mfma_bf16(a, uh[kk][s], O);
        O = mfma_bf16(a, ul[kk][s], O);
      }
    if (row_ok) {
#pragma unroll
      for (int m4 = 0; m4 < 4; m4++) {
        v4f o4;
#pragma unroll
        for (int jj = 0; jj < 4; jj++) o4[jj] = O[4 * m4 + jj];
        *(v4f*)&orow[32 * rb + 8 * m4 + 4 * g2] = o4;
      }
    }
  }
}

}  // namespace


hipError_t wsvd_launch_prefill_attn(const wsvd_layer_desc& d, const void* q, int nq, int n_after, const void* B_K, const void* B_V,
                                    const wsvd_cache& cache, void* out, hipStream_t s, const wsvd_paged_cache* paged) {
  if (d.latent_dtype != WSVD_I8 || d.factor_dtype != WSVD_BF16 || d.q_dtype != WSVD_BF16) return hipErrorNotSupported;
  if (d.d_head % 32 != 0 || nq < 1 || n_after < 0) return hipErrorInvalidValue;
  PrefillParams p;
  p.q = (const uint16_t*)q; p.BK = (const uint16_t*)B_K; p.BV = (const uint16_t*)B_V;
  p.k_codes = (const uint8_t*)cache.k_codes; p.v_codes = (const uint8_t*)cache.v_codes;
  p.k_meta = (const uint16_t*)cache.k_meta; p.v_meta = (const uint16_t*)cache.v_meta;
  p.seq_lens = cache.seq_lens; p.out = (float*)out;
  p.B = d.batch; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads; p.d = d.d_head; p.t_cap = d.t_cap;
  p.nq = nq; p.n_after = n_after;
  p.block_table = nullptr; p.page_rows = p.max_pages = p.n_pages = 0;
  if (paged) { p.block_table = paged->block_table; p.page_rows = paged->page_rows; p.max_pages = paged->max_pages; p.n_pages = paged->n_pages; }
  const int64_t NR = (int64_t)nq * p.G;
  if (NR > (int64_t)65535 * 32) return hipErrorInvalidValue;
  p.NR = (int)NR;
  const float sm = d.sm_scale != 0.f ? d.sm_scale : 1.0f / sqrtf((float)d.d_head);
  p.c_scale = sm * 1.44269504088896340736f;
  dim3 grid((unsigned)d.n_kv_heads, (unsigned)((NR + 31) / 32), (unsigned)d.batch);
  if (d.rank == 32) hipLaunchKernelGGL((k_prefill_attn<32>), grid, dim3(64), 0, s, p);
  else if (d.rank == 64) hipLaunchKernelGGL((k_prefill_attn<64>), grid, dim3(64), 0, s, p);
  else return hipErrorNotSupported;
  return hipGetLastError();
}
