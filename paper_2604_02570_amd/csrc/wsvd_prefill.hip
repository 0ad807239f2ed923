// Causal attention of a block of query tokens over the int8 latent cache, tiled for the matrix cores (the attention
// of prefilling, Section 3.4, in latent space).
//
// With no rotation between the reconstruction and the product, q K^T = (q B_K^T) C_K^T and P V = (P C_V) B_V: the
// whole score / softmax / value loop runs on latents of dimension r instead of keys and values of dimension d.
//   prologue  Q~^T [r x 32 queries] = B_K q^T                       bf16 MFMA, operands straight from global memory
//   loop      S^T [32 keys x 32 queries] = C_K Q~^T                 fp16 MFMA: codes are exact in fp16, Q~ is an fp16 pair
//             online softmax down the columns (a lane owns one query column: running max and sum are per lane)
//             U^T [r x 32 queries] += C_V^T (P diag(s_V))           bf16 MFMA: codes exact, P an bf16 pair, through LDS
//   epilogue  O^T [d x 32 queries] = B_V^T (U / l)                  bf16 MFMA, U an bf16 pair
// One wavefront per (sequence, kv head, block of 32 query rows); a query row is a (token, head) pair, token-major, so
// the G heads that share a kv head share the stream too.  The cache blocks are read in the layout the decode kernels
// use (a 32-token block of the K plane is a ready-made operand with row = token, one of the V plane with row = dim).
// 32x32 accumulator layout throughout: lane L holds column L % 32, rows 8 (v / 4) + 4 (L / 32) + v % 4, v = 0..15.
#include "wsvd_dev.h"
#include "wsvd_internal.h"

namespace {

typedef __bf16 v8bf16 __attribute__((ext_vector_type(8)));
typedef _Float16 v8f16 __attribute__((ext_vector_type(8)));

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
};

WSVD_DEV v16f mfma_bf16(v8bf16 a, v8bf16 b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
WSVD_DEV v16f mfma_f16(v8f16 a, v8f16 b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }

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

// 8 int8 codes (two dwords) -> 8 fp16 / bf16 operand elements, exact
WSVD_DEV v8f16 codes_f16(int d0, int d1) {
  v8f16 r;
#pragma unroll
  for (int e = 0; e < 4; e++) { r[e] = (_Float16)(int)(int8_t)(d0 >> (8 * e)); r[4 + e] = (_Float16)(int)(int8_t)(d1 >> (8 * e)); }
  return r;
}
WSVD_DEV v8bf16 codes_bf16(int d0, int d1) {
  v4i r;
#pragma unroll
  for (int e = 0; e < 2; e++) {
    const uint32_t a0 = __float_as_uint((float)(int)(int8_t)(d0 >> (16 * e))) >> 16, a1 = __float_as_uint((float)(int)(int8_t)(d0 >> (16 * e + 8))) & 0xFFFF0000u;
    const uint32_t b0 = __float_as_uint((float)(int)(int8_t)(d1 >> (16 * e))) >> 16, b1 = __float_as_uint((float)(int)(int8_t)(d1 >> (16 * e + 8))) & 0xFFFF0000u;
    r[e] = (int)(a0 | a1);
    r[2 + e] = (int)(b0 | b1);
  }
  return __builtin_bit_cast(v8bf16, r);
}

template <int R>
__global__ __launch_bounds__(64) void k_prefill_attn(PrefillParams p) {
  constexpr int KK = R / 32;
  __shared__ __attribute__((aligned(16))) float sc_lds[2][32];          // K and V scales of the block's 32 tokens
  __shared__ __attribute__((aligned(16))) uint16_t pt[2][32][40];       // P diag(s_V) as a bf16 pair, [query][key], padded rows

  const int lane = threadIdx.x, n = lane & 31, g2 = lane >> 5;
  const int kv = blockIdx.x, qb = blockIdx.y, b = blockIdx.z;
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

  // one block ahead in registers
  v4i kc[KK], vc[KK];
  uint16_t ks_raw, vs_raw;
  auto load_block = [&](int kb) {
    const size_t off = (size_t)kb * (32 * R) + (size_t)lane * 16;
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      kc[kk] = __builtin_nontemporal_load((const v4i*)(kplane + off + kk * 1024));
      vc[kk] = __builtin_nontemporal_load((const v4i*)(vplane + off + kk * 1024));
    }
    ks_raw = kmeta[kb * 32 + n];
    vs_raw = vmeta[kb * 32 + n];
  };
  load_block(0);

  for (int kb = 0; kb < n_kblocks; kb++) {
    // this block's operands out of the load registers, then the next block's loads
    v8f16 aK[2 * KK];
    v8bf16 aV[KK][2];
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      aK[2 * kk] = codes_f16(kc[kk][0], kc[kk][1]);
      aK[2 * kk + 1] = codes_f16(kc[kk][2], kc[kk][3]);
      aV[kk][0] = codes_bf16(vc[kk][0], vc[kk][1]);
      aV[kk][1] = codes_bf16(vc[kk][2], vc[kk][3]);
    }
    if (g2 == 0) { sc_lds[0][n] = f16_bits_to_f32(ks_raw); sc_lds[1][n] = f16_bits_to_f32(vs_raw); }
    if (kb + 1 < n_kblocks) load_block(kb + 1);

    // scores of the block: rows = its 32 tokens, columns = the 32 queries
    v16f S;
#pragma unroll
    for (int v = 0; v < 16; v++) S[v] = 0.f;
#pragma unroll
    for (int s = 0; s < 2 * KK; s++) { S = mfma_f16(aK[s], qh[s], S); S = mfma_f16(aK[s], ql[s], S); }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float sk[16], sv[16];
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      const v4f k4 = *(const v4f*)&sc_lds[0][8 * m4 + 4 * g2], v4 = *(const v4f*)&sc_lds[1][8 * m4 + 4 * g2];
#pragma unroll
      for (int jj = 0; jj < 4; jj++) { sk[4 * m4 + jj] = k4[jj]; sv[4 * m4 + jj] = v4[jj]; }
    }
    float sc[16];
    float bmax = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; v++) {
      const int key = kb * 32 + 8 * (v >> 2) + 4 * g2 + (v & 3);
      sc[v] = key < lim ? S[v] * sk[v] : -INFINITY;
      bmax = fmaxf(bmax, sc[v]);
    }
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32));                           // the other half holds the column's other rows
    const float m_new = fmaxf(m_run, bmax);
    const float alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.f;
    float pw[16];
#pragma unroll
    for (int v = 0; v < 16; v++) {
      pw[v] = sc[v] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sc[v] - m_new);
      psum += pw[v];
    }
    l_run = fmaf(l_run, alpha, psum);
    m_run = m_new;
#pragma unroll
    for (int kk = 0; kk < KK; kk++)
#pragma unroll
      for (int v = 0; v < 16; v++) U[kk][v] *= alpha;
    // P diag(s_V) as a bf16 pair -> LDS, [query][key]: a lane's 16 rows are 4 runs of 4 consecutive keys
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int jj = 0; jj < 4; jj++)      // a hidden row's scale may be anything (never-written rows): keep it out
        split_bf16(pw[4 * m4 + jj] == 0.f ? 0.f : pw[4 * m4 + jj] * sv[4 * m4 + jj], hi[jj], lo[jj]);
      v2i ph2, pl2;
      ph2[0] = (int)((hi[0] >> 16) | hi[1]); ph2[1] = (int)((hi[2] >> 16) | hi[3]);
      pl2[0] = (int)((lo[0] >> 16) | lo[1]); pl2[1] = (int)((lo[2] >> 16) | lo[3]);
      *(v2i*)&pt[0][n][8 * m4 + 4 * g2] = ph2;
      *(v2i*)&pt[1][n][8 * m4 + 4 * g2] = pl2;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // U^T += C_V^T P: rows = latent dims, columns = queries; step s contracts the tokens 16 g2 + 8 s .. + 7 of a half
#pragma unroll
    for (int s = 0; s < 2; s++) {
      const v8bf16 bh = *(const v8bf16*)&pt[0][n][16 * g2 + 8 * s], bl = *(const v8bf16*)&pt[1][n][16 * g2 + 8 * s];
#pragma unroll
      for (int kk = 0; kk < KK; kk++) { U[kk] = mfma_bf16(aV[kk][s], bh, U[kk]); U[kk] = mfma_bf16(aV[kk][s], bl, U[kk]); }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

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

// ---------------------------------------------------------------- cache build for a whole prompt (int8 latents)
// C^T [channels x tokens] = A^T x^T on bf16 MFMA.  The channels of both planes form one axis of 2 * Hkv * r / 32 tiles
// of 32; a wavefront owns CT channel tiles x TT token tiles (CT * TT accumulators of 32 x 32), so each 1 KiB operand it
// fetches feeds CT or TT products.  The A operand is the packed factor image the append kernels use (1 KiB per
// 32 channels x 16 model dims, contiguous); the B operand is 16 bytes of a token's hidden state per lane.  The 4 waves
// of a workgroup take 4 neighbouring channel groups of the same tokens, so the hidden states come out of the CU's
// first-level cache after the first wave; operands are requested ST - 1 steps ahead of the products that use them.
// A lane ends up with 16 of every 32 channels of ITS tokens (the other half wave holds the rest): the per-token scale of
// a head is a maximum over registers plus one exchange, and the codes go out in the decode layout (4 consecutive
// channels of a K row are 4 adjacent bytes; a V row is written byte by byte, its neighbours in a 16-byte group being
// other tokens).
struct ProjectParams {
  const uint16_t* x;          // bf16 [n_seq, n_tok, E]
  const uint16_t* A[2];       // packed factors
  uint8_t* codes[2];
  uint16_t* meta[2];
  int* seq_lens;
  int* err_word;
  int Hkv, E, t_cap, n_tok, seq0;   // direct kernel: grid z = sequence - seq0
  int n_cg, tg_seq, n_tg;           // staged kernel: channel groups, token groups per sequence and in all
};

// per token and head: symmetric int8 (the latent quantiser's rule), then the stores.  acc[c][tt] = channel tile ct0 + c
// x token tile tb * TT + tt of this wave, in the 32 x 32 accumulator order.
template <int R, int CT, int TT>
WSVD_DEV void project_store(const ProjectParams& p, v16f (&acc)[CT][TT], int ct0, int tb, int seq, int n0) {
  constexpr int RT = R / 32;
  const int lane = threadIdx.x & 63, n = lane & 31, g2 = lane >> 5;
  const int tiles_plane = p.Hkv * RT, tiles = 2 * tiles_plane;
#pragma unroll
  for (int h = 0; h < CT / RT; h++) {
    const int ct = ct0 + h * RT;
    if (ct >= tiles) break;
    const int pl = ct / tiles_plane, kv = (ct % tiles_plane) / RT;
    const size_t ph = (size_t)seq * p.Hkv + kv;
    uint8_t* plane = p.codes[pl] + ph * (size_t)p.t_cap * R;
#pragma unroll
    for (int tt = 0; tt < TT; tt++) {
      float a = 0.f;
#pragma unroll
      for (int rt = 0; rt < RT; rt++)
#pragma unroll
        for (int v = 0; v < 16; v++) a = fmaxf(a, fabsf(acc[h * RT + rt][tt][v]));
      a = fmaxf(a, __shfl_xor(a, 32));
      uint16_t sh = 0x3C00u;
      if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
      const float sc = f16_bits_to_f32(sh);
      const int tok = (tb * TT + tt) * 32 + n;                          // this lane's token of the prompt
      const int t = n0 + tok;                                           // and its cache row
      if (tok >= p.n_tok || n0 < 0 || t >= p.t_cap) continue;
#pragma unroll
      for (int rt = 0; rt < RT; rt++)
#pragma unroll
        for (int m4 = 0; m4 < 4; m4++) {
          uint32_t pk = 0;
          int q[4];
#pragma unroll
          for (int jj = 0; jj < 4; jj++) {
            q[jj] = (int)fminf(fmaxf(__builtin_rintf(acc[h * RT + rt][tt][4 * m4 + jj] / sc), -127.f), 127.f);
            pk |= ((uint32_t)q[jj] & 0xFFu) << (8 * jj);
          }
          const int j0 = 32 * rt + 8 * m4 + 4 * g2;                     // channels j0 .. j0 + 3
          if (pl == 0) *(uint32_t*)(plane + i8_k_offset(t, j0, R)) = pk;
          else {
#pragma unroll
            for (int jj = 0; jj < 4; jj++) plane[i8_v_offset(t, j0 + jj, R)] = (uint8_t)q[jj];
          }
        }
      if (g2 == 0) p.meta[pl][ph * p.t_cap + t] = sh;
    }
  }
}

template <int R, int CT, int TT, int WC, int ST = 3>
__global__ __launch_bounds__(256) void k_prefill_project(ProjectParams p) {
  constexpr int RT = R / 32;
  static_assert(CT % RT == 0, "a head's channels stay in one wave");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, g2 = lane >> 5;
  const int tiles_plane = p.Hkv * RT, tiles = 2 * tiles_plane;
  const int ct0 = (blockIdx.x * WC + wave % WC) * CT;                   // first channel tile of this wave
  const int tb = blockIdx.y * (4 / WC) + wave / WC;                     // its group of TT token tiles
  if (ct0 >= tiles || tb * 32 * TT >= p.n_tok) return;
  const int seq = p.seq0 + blockIdx.z;
  const int n0 = p.seq_lens[seq];
  const int n_steps = p.E >> 4;
  const uint16_t* ap[CT];
#pragma unroll
  for (int c = 0; c < CT; c++) {
    const int ct = min(ct0 + c, tiles - 1);
    ap[c] = p.A[ct / tiles_plane] + ((size_t)(ct % tiles_plane) * n_steps * 64 + lane) * 8;
  }
  const uint16_t* xp[TT];
#pragma unroll
  for (int tt = 0; tt < TT; tt++) {
    const int tok = min((tb * TT + tt) * 32 + n, p.n_tok - 1);
    xp[tt] = p.x + ((size_t)blockIdx.z * p.n_tok + tok) * p.E + 8 * g2;
  }
  v16f acc[CT][TT];
#pragma unroll
  for (int c = 0; c < CT; c++)
#pragma unroll
    for (int tt = 0; tt < TT; tt++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[c][tt][v] = 0.f;
  v8bf16 fa[ST][CT], fb[ST][TT];
  auto fetch = [&](int st, int ks) {
    ks = min(ks, n_steps - 1);
#pragma unroll
    for (int c = 0; c < CT; c++) fa[st][c] = *(const v8bf16*)(ap[c] + (size_t)ks * 512);
#pragma unroll
    for (int tt = 0; tt < TT; tt++) fb[st][tt] = *(const v8bf16*)(xp[tt] + 16 * ks);
  };
#pragma unroll
  for (int u = 0; u < ST - 1; u++) fetch(u, u);
  for (int ks0 = 0; ks0 < n_steps; ks0 += ST) {
#pragma unroll
    for (int u = 0; u < ST; u++) {
      fetch((u + ST - 1) % ST, ks0 + u + ST - 1);
      if (ks0 + u < n_steps) {
#pragma unroll
        for (int c = 0; c < CT; c++)
#pragma unroll
          for (int tt = 0; tt < TT; tt++) acc[c][tt] = mfma_bf16(fa[u][c], fb[u][tt], acc[c][tt]);
      }
    }
  }
  project_store<R, CT, TT>(p, acc, ct0, tb, seq, n0);
}

// The same projection with both operands staged through LDS: a workgroup of 4 waves (2 x 2, each 4 x 4 tiles) owns
// 256 channels x 256 tokens.  Per chunk of 64 model dims it copies 32 KiB of the factor image (already in operand order)
// and 256 whole 128-byte lines of hidden states (rows padded to 144 bytes in LDS, which makes the operand reads free of
// bank conflicts), so that the first-level cache sees whole lines once per workgroup instead of 32-byte pieces once per
// wave.  Two LDS stages: the next chunk travels global -> registers during the products of the current one and is
// written to the other stage before the chunk's only barrier.  E must be a multiple of 64.
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
constexpr int kProjKC = 64, kProjXRow = 144;
constexpr int kProjABytes = 8 * 4 * 1024, kProjXBytes = 256 * kProjXRow, kProjStage = kProjABytes + kProjXBytes;

template <int R>
__global__ __launch_bounds__(256) void k_prefill_project_lds(ProjectParams p) {
  extern __shared__ __align__(16) uint8_t proj_lds[];
  constexpr int RT = R / 32, CT = 4, TT = 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, g2 = lane >> 5;
  const int wc = wave & 1, wt = wave >> 1;
  const int tiles_plane = p.Hkv * RT, tiles = 2 * tiles_plane;
  // Workgroup -> (channel group, token group).  Consecutive workgroup ids land on different XCDs (8 of them, each with
  // its own L2): when the number of token groups allows it, XCD i takes the token groups = i (mod 8), so a line of hidden
  // states is fetched by one XCD only, and the workgroups running together on an XCD cover all channel groups of a few
  // token groups, walking through the factors in step.
  int cg, tg;
  {
    const int L = blockIdx.x;
    if (p.n_tg % 8 == 0) { const int sl = L >> 3; cg = sl % p.n_cg; tg = (sl / p.n_cg) * 8 + (L & 7); }
    else { cg = L % p.n_cg; tg = L / p.n_cg; }
  }
  const int sq = tg / p.tg_seq, by = tg % p.tg_seq;                     // sequence of the launch, 256-token group in it
  const int seq = p.seq0 + sq;
  const int n0 = p.seq_lens[seq];
  const int n_steps = p.E >> 4, n_chunks = p.E / kProjKC;
  // what this thread copies per chunk: 16 bytes of each of the 8 channel tiles, 16 bytes of 8 of the 256 token rows
  // (uniform base pointers plus 32-bit per-thread offsets: the loads address through scalar registers)
  const uint8_t* asrc[8];
  const uint8_t* xbase = (const uint8_t*)p.x + (size_t)sq * p.n_tok * p.E * 2;
  uint32_t xoff[8];
  int xdst[8];
  const uint32_t aoff = tid * 16;
#pragma unroll
  for (int j = 0; j < 8; j++) {
    const int ct = min(cg * 8 + j, tiles - 1);
    asrc[j] = (const uint8_t*)p.A[ct / tiles_plane] + (size_t)(ct % tiles_plane) * n_steps * 1024;
    const int u = tid + 256 * j, row = u >> 3, sg = u & 7;
    const int tok = min(by * 256 + row, p.n_tok - 1);
    xoff[j] = (uint32_t)tok * (uint32_t)(p.E * 2) + sg * 16;            // the launcher keeps n_tok * E * 2 below 2^31
    xdst[j] = kProjABytes + row * kProjXRow + sg * 16;
  }
  v4u rg[16];                                                           // the chunk on its way: 8 pieces of A, 8 of x
  auto fetch1 = [&](int j, int c) {
    c = min(c, n_chunks - 1);                     // (past the end: the last chunk again, written to the idle stage, never read)
    if (j < 8) rg[j] = *(const v4u*)(asrc[j] + (size_t)c * 4096 + aoff);
    else rg[j] = *(const v4u*)(xbase + (size_t)c * (kProjKC * 2) + xoff[j - 8]);
  };
  auto commit1 = [&](int j, int st) {
    uint8_t* base = proj_lds + st * kProjStage;
    if (j < 8) *(v4u*)(base + j * 4096 + tid * 16) = rg[j];
    else *(v4u*)(base + xdst[j - 8]) = rg[j];
  };
  v16f acc[CT][TT];
#pragma unroll
  for (int c = 0; c < CT; c++)
#pragma unroll
    for (int tt = 0; tt < TT; tt++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[c][tt][v] = 0.f;
  const int a_off = wc * 4 * 4096 + lane * 16;                          // + c * 4096 + ks * 1024
  const int x_off = kProjABytes + (wt * 128 + n) * kProjXRow + g2 * 16; // + tt * 32 rows + ks * 32 bytes
#pragma unroll
  for (int j = 0; j < 16; j++) fetch1(j, 0);
#pragma unroll
  for (int j = 0; j < 16; j++) commit1(j, 0);
  __syncthreads();
  // One wave per SIMD: nothing else fills the issue slots this wave leaves empty, so the order of its instructions is
  // fixed by hand.  Per step of 16 model dims: the 8 operand reads of the NEXT step, then 4 groups of 4 products, each
  // followed, in the first two steps, by two 16-byte requests of the next chunk and, in the last step, by four 16-byte
  // writes of it to the idle stage: requests and writes trickle into the memory pipelines between products instead of
  // blocking the wave in a burst.
  for (int c = 0; c < n_chunks; c++) {
    const uint8_t* base = proj_lds + (c & 1) * kProjStage;
    v8bf16 fa[2][CT], fb[2][TT];
    auto frags = [&](int b, int ks) {
#pragma unroll
      for (int cc = 0; cc < CT; cc++) fa[b][cc] = *(const v8bf16*)(base + a_off + cc * 4096 + ks * 1024);
#pragma unroll
      for (int tt = 0; tt < TT; tt++) fb[b][tt] = *(const v8bf16*)(base + x_off + tt * 32 * kProjXRow + ks * 32);
    };
    frags(0, 0);
#pragma unroll
    for (int ks = 0; ks < kProjKC / 16; ks++) {
      if (ks + 1 < kProjKC / 16) frags((ks + 1) & 1, ks + 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int cc = 0; cc < CT; cc++) {
#pragma unroll
        for (int tt = 0; tt < TT; tt++) acc[cc][tt] = mfma_bf16(fa[ks & 1][cc], fb[ks & 1][tt], acc[cc][tt]);
        __builtin_amdgcn_sched_barrier(0);
        if (ks < 2) { fetch1(2 * (ks * 4 + cc), c + 1); fetch1(2 * (ks * 4 + cc) + 1, c + 1); }
        if (ks == 3) {
#pragma unroll
          for (int j = 0; j < 4; j++) commit1(4 * cc + j, (c + 1) & 1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
  }
  const int ct0 = (cg * 2 + wc) * CT, tb = by * 2 + wt;
  if (ct0 >= tiles || tb * 32 * TT >= p.n_tok) return;
  project_store<R, CT, TT>(p, acc, ct0, tb, seq, n0);
}

// after the projection: the lengths move on by the rows that fitted (one thread per sequence)
__global__ void k_prefill_bump(int* seq_lens, int seq0, int n_seq, int n_tok, int t_cap, int* err_word) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_seq) return;
  const int n0 = seq_lens[seq0 + i];
  if (n0 >= 0) seq_lens[seq0 + i] = min(n0 + n_tok, t_cap);
  if (n0 < 0 || n0 + n_tok > t_cap) atomicExch(err_word, (int)WSVD_E_CAPACITY);
}

template <int R, int CT, int TT, int WC, int ST = 3>
void launch_project(const ProjectParams& p, int n_seq, hipStream_t s) {
  const int tiles = 2 * p.Hkv * (R / 32), tok_wg = 32 * TT * (4 / WC);
  dim3 grid((unsigned)((tiles + WC * CT - 1) / (WC * CT)), (unsigned)((p.n_tok + tok_wg - 1) / tok_wg), (unsigned)n_seq);
  hipLaunchKernelGGL((k_prefill_project<R, CT, TT, WC, ST>), grid, dim3(256), 0, s, p);
}

}  // namespace

int g_wsvd_project_shape = 0;

hipError_t wsvd_launch_prefill_project(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, int n_tok, int seq,
                                       const void* A_K, const void* A_V, const wsvd_cache& cache, hipStream_t s) {
  if (d.latent_dtype != WSVD_I8 || d.factor_dtype != WSVD_BF16 || d.x_dtype != WSVD_BF16) return hipErrorNotSupported;
  if (d.rank != 32 && d.rank != 64) return hipErrorNotSupported;
  if (d.d_model % 16 != 0 || n_tok < 1) return hipErrorInvalidValue;
  ProjectParams p;
  p.x = (const uint16_t*)x; p.A[0] = (const uint16_t*)A_K; p.A[1] = (const uint16_t*)A_V;
  p.codes[0] = (uint8_t*)cache.k_codes; p.codes[1] = (uint8_t*)cache.v_codes;
  p.meta[0] = (uint16_t*)cache.k_meta; p.meta[1] = (uint16_t*)cache.v_meta;
  p.seq_lens = cache.seq_lens; p.err_word = ctx->err_word;
  p.Hkv = d.n_kv_heads; p.E = d.d_model; p.t_cap = d.t_cap; p.n_tok = n_tok;
  p.n_cg = p.tg_seq = p.n_tg = 0;
  const int n_seq = seq < 0 ? d.batch : 1;
  p.seq0 = seq < 0 ? 0 : seq;
  // small problems: small wave tiles, so that there are enough waves; prompt-sized ones: the LDS-staged kernel
  // (option "project_shape": 1 = staged, 44 / 42 / 24 / 21 = variants of the direct kernel, for tuning and tests)
  const long long work = (long long)n_seq * n_tok * d.n_kv_heads * d.rank;
  const bool staged_ok = d.d_model % kProjKC == 0 && (long long)n_tok * d.d_model * 2 < (1LL << 31);
  int shape = g_wsvd_project_shape ? g_wsvd_project_shape : (work >= (1LL << 22) ? (staged_ok ? 1 : 44) : 21);
  if (shape == 1 && !staged_ok) shape = 44;
  if (shape == 1) {
    const int tiles = 2 * p.Hkv * (d.rank / 32);
    p.n_cg = (tiles + 7) / 8; p.tg_seq = (n_tok + 255) / 256; p.n_tg = p.tg_seq * n_seq;
    dim3 grid((unsigned)(p.n_cg * p.n_tg));
    const size_t lds = 2 * (size_t)kProjStage;
    static bool raised[2] = {false, false};              // the kernels' limit of dynamic LDS, raised once
    const void* fn = d.rank == 32 ? (const void*)k_prefill_project_lds<32> : (const void*)k_prefill_project_lds<64>;
    if (!raised[d.rank == 64]) {
      hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      raised[d.rank == 64] = true;
    }
    if (d.rank == 32) hipLaunchKernelGGL((k_prefill_project_lds<32>), grid, dim3(256), lds, s, p);
    else hipLaunchKernelGGL((k_prefill_project_lds<64>), grid, dim3(256), lds, s, p);
  } else if (d.rank == 32) {
    if (shape == 44) launch_project<32, 4, 4, 4>(p, n_seq, s);
    else if (shape == 42) launch_project<32, 4, 4, 4, 4>(p, n_seq, s);
    else if (shape == 24) launch_project<32, 4, 4, 4, 6>(p, n_seq, s);
    else launch_project<32, 2, 1, 4>(p, n_seq, s);
  } else {
    if (shape == 44) launch_project<64, 4, 4, 4>(p, n_seq, s);
    else if (shape == 42) launch_project<64, 4, 4, 2>(p, n_seq, s);
    else if (shape == 24) launch_project<64, 4, 4, 1>(p, n_seq, s);
    else launch_project<64, 2, 1, 4>(p, n_seq, s);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_prefill_bump, dim3((n_seq + 63) / 64), dim3(64), 0, s, cache.seq_lens, p.seq0, n_seq, n_tok, d.t_cap, ctx->err_word);
  return hipGetLastError();
}

int g_wsvd_prefill_tiled = 0;

hipError_t wsvd_launch_prefill_attn(const wsvd_layer_desc& d, const void* q, int nq, int n_after, const void* B_K, const void* B_V,
                                    const wsvd_cache& cache, void* out, hipStream_t s) {
  if (d.latent_dtype != WSVD_I8 || d.factor_dtype != WSVD_BF16 || d.q_dtype != WSVD_BF16) return hipErrorNotSupported;
  if (d.d_head % 32 != 0 || nq < 1 || n_after < 0) return hipErrorInvalidValue;
  PrefillParams p;
  p.q = (const uint16_t*)q; p.BK = (const uint16_t*)B_K; p.BV = (const uint16_t*)B_V;
  p.k_codes = (const uint8_t*)cache.k_codes; p.v_codes = (const uint8_t*)cache.v_codes;
  p.k_meta = (const uint16_t*)cache.k_meta; p.v_meta = (const uint16_t*)cache.v_meta;
  p.seq_lens = cache.seq_lens; p.out = (float*)out;
  p.B = d.batch; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads; p.d = d.d_head; p.t_cap = d.t_cap;
  p.nq = nq; p.n_after = n_after;
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
