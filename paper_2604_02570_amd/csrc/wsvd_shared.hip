// Decode attention over ONE shared rank-R latent per token with per-head up-projections: the conventional whole-matrix
// scheme the per-head method is contrasted with (Section 3.1, panel (b) of its figure; the "W/o per-head" variant of the
// latency appendix).  Built here in the form that suits the matrix cores: with the up-projection absorbed into the query,
// the 32 heads are the columns of a GEMM over the shared latent,
//     S [tokens x heads] = C_K [tokens x R] Q~^T [R x heads],     U^T [R x heads] += (diag(s_V) C_V)^T P [tokens x heads],
// so the latent stream is read ONCE for all heads (not once per head, as a per-head kernel run on the shared latent
// would), at the price of R-dimensional per-head queries and outputs: Q~_h = B_Kh q_h and o_h = B_Vh^T u_h move
// 2 * H * R * d factor elements per step where the per-head scheme moves 2 * H * r * d.
//   k_shared_absorb   Q~ [B, H, R] = (sm_scale log2 e) B_Kh q_h              bf16 MFMA, one wave per (head, 32 latent dims)
//   k_shared_attn     per (sequence, split of its 128-token chunks): scores on int8 MFMA (the cache codes are the A
//                     operand as stored; Q~ as three 7-bit limbs in LDS is the B operand), softmax down the head
//                     columns, value product on fp16 MFMA with each wave owning a quarter of the R output dims;
//                     partial (m, l, U) per split
//   k_shared_out      merge of the splits, u = U / l, o_h = B_Vh^T u_h         vector ALU, one workgroup per (head, sequence)
// 32x32 accumulator layout throughout: lane L holds column L % 32, rows 8 (v / 4) + 4 (L / 32) + v % 4, v = 0..15.
#include "wsvd_dev.h"
#include "wsvd_internal.h"

namespace {

constexpr int kSharedHeads = 32;          // the heads are the 32 columns of the products
constexpr int kSharedChunk = 128;         // tokens per workgroup pass: one 32-token block per wave
constexpr float kLimbRange = 1040000.f;   // |Q~ / delta| stays below 2^20: three signed 7-bit limbs

struct SharedParams {
  const uint16_t* q;          // bf16 [B, H, d]
  const uint16_t* BK;         // bf16 [H, R, d]
  const uint16_t* BV;
  const uint8_t* k_codes;     // [B][t_cap * R], 32-token blocks
  const uint8_t* v_codes;
  const uint16_t* k_scale;    // fp16 [B][t_cap]
  const uint16_t* v_scale;
  const int* seq_lens;
  float* qt;                  // workspace: Q~ [B, H, R]
  float* qmax;                //            max |Q~| per (sequence, head) (ranks above 1024 only)
  float* pm;                  // workspace: partial running maxima [B, S, H]
  float* pl;                  //            partial sums           [B, S, H]
  float* pu;                  //            partial U              [B, S, H, R]
  float* out;                 // fp32 [B, H, d]
  int B, d, R, t_cap, S;
  int per;                    // chunks of 128 tokens per split (ranks above 1024: at most 4)
  float c_scale;              // sm_scale * log2(e)
};

// ---------------------------------------------------------------- Q~ = c B_Kh q_h
__global__ __launch_bounds__(64) void k_shared_absorb(SharedParams p) {
  const int lane = threadIdx.x, n = lane & 31, g2 = lane >> 5;
  const int jb = blockIdx.x, h = blockIdx.y;
  const uint16_t* arow = p.BK + ((size_t)h * p.R + 32 * jb + n) * p.d + 8 * g2;
  for (int bb = 0; bb < p.B; bb += 32) {
    const int b = bb + n;
    const uint16_t* qrow = p.q + ((size_t)min(b, p.B - 1) * kSharedHeads + h) * p.d + 8 * g2;
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] = 0.f;
    for (int ks = 0; ks < (p.d >> 4); ks++)
      acc = mfma_bf16(*(const v8bf16*)(arow + 16 * ks), *(const v8bf16*)(qrow + 16 * ks), acc);
    if (b < p.B) {
      float* dst = p.qt + ((size_t)b * kSharedHeads + h) * p.R + 32 * jb + 4 * g2;
#pragma unroll
      for (int m4 = 0; m4 < 4; m4++) {
        v4f o;
#pragma unroll
        for (int jj = 0; jj < 4; jj++) o[jj] = acc[4 * m4 + jj] * p.c_scale;
        *(v4f*)(dst + 8 * m4) = o;
      }
    }
  }
}

// ---------------------------------------------------------------- attention over the shared latent, all heads at once
// LDS: limbs [3][R / 32][64 lanes][16 B], then 4 float tables [4 waves][32], then P tiles [4 waves][32 heads][40] fp16.
template <int R>
__global__ __launch_bounds__(256) void k_shared_attn(SharedParams p) {
  constexpr int NKS = R / 32;             // 32-dim steps of the score contraction
  constexpr int NKK = R / 128;            // 32-dim sub-blocks of the value dims one wave owns
  extern __shared__ __align__(16) uint8_t sh_lds[];
  v4i* limbs = (v4i*)sh_lds;                                            // [3][NKS][64]
  float* hmax = (float*)(sh_lds + 3 * NKS * 1024);                      // [4][32] each
  float* cmax = hmax + 128;
  float* csum = cmax + 128;
  float* ksc = csum + 128;
  _Float16* pt = (_Float16*)(ksc + 128);                                // [4][32][40]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, g2 = lane >> 5;
  const int split = blockIdx.x, b = blockIdx.y;
  const int n_b = min(max(p.seq_lens[b], 0), p.t_cap);
  const int n_chunks = (n_b + kSharedChunk - 1) / kSharedChunk;
  const int per = (n_chunks + p.S - 1) / p.S;
  const int c0 = split * per, c1 = min(c0 + per, n_chunks);
  const size_t part = (size_t)b * p.S + split;
  if (c0 >= c1) {                                                       // nothing for this split: the merge skips it
    if (tid < kSharedHeads) { p.pm[part * kSharedHeads + tid] = -INFINITY; p.pl[part * kSharedHeads + tid] = 0.f; }
    return;
  }

  const uint8_t* kplane = p.k_codes + (size_t)b * p.t_cap * R;
  const uint8_t* vplane = p.v_codes + (size_t)b * p.t_cap * R;
  const uint16_t* kmeta = p.k_scale + (size_t)b * p.t_cap;
  const uint16_t* vmeta = p.v_scale + (size_t)b * p.t_cap;

  // ---- Q~ of head n as three signed 7-bit limbs of round(Q~ / delta_n): lane (n, g2) of step ks holds dims
  // 32 ks + 16 g2 .. + 15, the B operand of the int8 product as it is
  const float* qrow = p.qt + ((size_t)b * kSharedHeads + n) * R + 16 * g2;
  constexpr int NQ = NKS / 4;                                           // steps this wave converts
  v4f xq[NQ][4];                                                        // read once, all requests in flight together
#pragma unroll
  for (int i = 0; i < NQ; i++)
#pragma unroll
    for (int i4 = 0; i4 < 4; i4++) xq[i][i4] = *(const v4f*)(qrow + 32 * (wave + 4 * i) + 4 * i4);
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < NQ; i++)
#pragma unroll
    for (int i4 = 0; i4 < 4; i4++)
      amax = fmaxf(amax, fmaxf(fmaxf(fabsf(xq[i][i4][0]), fabsf(xq[i][i4][1])), fmaxf(fabsf(xq[i][i4][2]), fabsf(xq[i][i4][3]))));
  amax = fmaxf(amax, __shfl_xor(amax, 32));
  if (g2 == 0) hmax[wave * 32 + n] = amax;
  __syncthreads();
  const float hm = fmaxf(fmaxf(hmax[n], hmax[32 + n]), fmaxf(hmax[64 + n], hmax[96 + n]));
  const float delta = hm > 0.f ? hm / kLimbRange : 1.0f;                // value of one unit of the integer query
  const float inv_delta = 1.0f / delta;
#pragma unroll
  for (int i = 0; i < NQ; i++) {
    const int ks = wave + 4 * i;
    v4i l0, l1, l2;
#pragma unroll
    for (int i4 = 0; i4 < 4; i4++) {
      uint32_t w0 = 0, w1 = 0, w2 = 0;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const int Q = (int)__builtin_rintf(xq[i][i4][e] * inv_delta);
        const int a0 = ((Q + 64) & 127) - 64, Q1 = (Q - a0) >> 7;       // Q = a0 + 128 Q1 exactly
        const int a1 = ((Q1 + 64) & 127) - 64, a2 = (Q1 - a1) >> 7;
        w0 |= ((uint32_t)a0 & 0xFFu) << (8 * e);
        w1 |= ((uint32_t)a1 & 0xFFu) << (8 * e);
        w2 |= ((uint32_t)a2 & 0xFFu) << (8 * e);
      }
      l0[i4] = (int)w0; l1[i4] = (int)w1; l2[i4] = (int)w2;
    }
    limbs[(0 * NKS + ks) * 64 + lane] = l0;
    limbs[(1 * NKS + ks) * 64 + lane] = l1;
    limbs[(2 * NKS + ks) * 64 + lane] = l2;
  }
  __syncthreads();

  float m_run = -INFINITY, l_run = 0.f;                                 // of head n (every wave keeps its own copy)
  v16f U[NKK];                                                          // rows = this wave's dims, columns = heads
#pragma unroll
  for (int kk = 0; kk < NKK; kk++)
#pragma unroll
    for (int v = 0; v < 16; v++) U[kk][v] = 0.f;

  for (int c = c0; c < c1; c++) {
    // ---- scores of this wave's 32 tokens against all heads
    const int t0 = c * kSharedChunk + 32 * wave;
    if (g2 == 0) ksc[wave * 32 + n] = f16_bits_to_f32(kmeta[t0 + n]);
    v16i a0, a1, a2;
#pragma unroll
    for (int v = 0; v < 16; v++) { a0[v] = 0; a1[v] = 0; a2[v] = 0; }
    // the K operands of the chunk: all R / 32 requests of this wave's 32 tokens in flight together (one trip to memory
    // per chunk instead of one per batch)
    v4i ka[NKS];
    {
      const uint8_t* kp = kplane + (size_t)(t0 >> 5) * (32 * R) + (size_t)lane * 16;
#pragma unroll
      for (int ks = 0; ks < NKS; ks++) ka[ks] = __builtin_nontemporal_load((const v4i*)(kp + (size_t)ks * 1024));
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ks++) {
      a0 = mfma_i8(ka[ks], limbs[(0 * NKS + ks) * 64 + lane], a0);
      a1 = mfma_i8(ka[ks], limbs[(1 * NKS + ks) * 64 + lane], a1);
      a2 = mfma_i8(ka[ks], limbs[(2 * NKS + ks) * 64 + lane], a2);
      if ((ks & 3) == 3) __builtin_amdgcn_sched_barrier(0);             // keeps the limb reads from piling up in registers
    }
    // the chunk's value blocks are requested now, all at once: they arrive during the softmax
    const int cbase = c * kSharedChunk;
    v4i vc[4][NKK], vsr[4][2];
#pragma unroll
    for (int tw = 0; tw < 4; tw++) {
      const int tv = min(cbase + 32 * tw, (n_b - 1) & ~31);             // (a block past the end: the last one again, unused)
      const uint8_t* vp = vplane + (size_t)(tv >> 5) * (32 * R) + (size_t)(wave * NKK) * 1024 + (size_t)lane * 16;
#pragma unroll
      for (int kk = 0; kk < NKK; kk++) vc[tw][kk] = __builtin_nontemporal_load((const v4i*)(vp + kk * 1024));
      vsr[tw][0] = *(const v4i*)(vmeta + tv + 16 * g2);
      vsr[tw][1] = *(const v4i*)(vmeta + tv + 16 * g2 + 8);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float sc[16];
    float bmax = -INFINITY;
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      const v4f k4 = *(const v4f*)&ksc[wave * 32 + 8 * m4 + 4 * g2];
#pragma unroll
      for (int jj = 0; jj < 4; jj++) {
        const int v = 4 * m4 + jj;
        const float s = fmaf(16384.f, (float)a2[v], fmaf(128.f, (float)a1[v], (float)a0[v])) * delta * k4[jj];
        sc[v] = t0 + 8 * m4 + 4 * g2 + jj < n_b ? s : -INFINITY;        // rows past the sequence's end
        bmax = fmaxf(bmax, sc[v]);
      }
    }
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
    if (g2 == 0) cmax[wave * 32 + n] = bmax;
    __syncthreads();
    const float m_new = fmaxf(m_run, fmaxf(fmaxf(cmax[n], cmax[32 + n]), fmaxf(cmax[64 + n], cmax[96 + n])));
    const float alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);   // m_new is finite: the chunk has a row
    float pw[16], psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; v++) {
      pw[v] = sc[v] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sc[v] - m_new);
      psum += pw[v];
    }
    psum += __shfl_xor(psum, 32);
    if (g2 == 0) csum[wave * 32 + n] = psum;
    _Float16* ptw = pt + (wave * 32 + n) * 40;
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      v4f p4;
#pragma unroll
      for (int jj = 0; jj < 4; jj++) p4[jj] = pw[4 * m4 + jj];
      *(v2i*)&ptw[8 * m4 + 4 * g2] = __builtin_bit_cast(v2i, __builtin_convertvector(p4, v4f16));
    }
    __syncthreads();
    l_run = fmaf(l_run, alpha, (csum[n] + csum[32 + n]) + (csum[64 + n] + csum[96 + n]));
    m_run = m_new;

    // ---- value product: this wave's quarter of the R dims, all four token blocks of the chunk
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int kk = 0; kk < NKK; kk++)
#pragma unroll
        for (int v = 0; v < 16; v++) U[kk][v] *= alpha;
    }
#pragma unroll
    for (int tw = 0; tw < 4; tw++) {
      const int tv = cbase + 32 * tw;
      if (tv < n_b) {
        v8f16 sv8[2] = {__builtin_bit_cast(v8f16, vsr[tw][0]), __builtin_bit_cast(v8f16, vsr[tw][1])};
        if (tv + 32 > n_b) {      // rows never written may hold any scale: they contribute 0
#pragma unroll
          for (int s = 0; s < 2; s++)
#pragma unroll
            for (int e = 0; e < 8; e++)
              if (tv + 16 * g2 + 8 * s + e >= n_b) sv8[s][e] = (_Float16)0;
        }
        const v8f16 bp0 = *(const v8f16*)&pt[(tw * 32 + n) * 40 + 16 * g2];
        const v8f16 bp1 = *(const v8f16*)&pt[(tw * 32 + n) * 40 + 16 * g2 + 8];
#pragma unroll
        for (int kk = 0; kk < NKK; kk++) {
          U[kk] = mfma_f16(codes_f16(vc[tw][kk][0], vc[tw][kk][1]) * sv8[0], bp0, U[kk]);
          U[kk] = mfma_f16(codes_f16(vc[tw][kk][2], vc[tw][kk][3]) * sv8[1], bp1, U[kk]);
        }
      }
    }
    __syncthreads();                                                    // the tables and P tiles are reused by the next chunk
  }

  // ---- partial result of this split
  if (wave == 0 && g2 == 0) { p.pm[part * kSharedHeads + n] = m_run; p.pl[part * kSharedHeads + n] = l_run; }
  float* pu = p.pu + (part * kSharedHeads + n) * R + (size_t)(wave * NKK) * 32 + 4 * g2;
#pragma unroll
  for (int kk = 0; kk < NKK; kk++)
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      v4f o;
#pragma unroll
      for (int jj = 0; jj < 4; jj++) o[jj] = U[kk][4 * m4 + jj];
      *(v4f*)(pu + 32 * kk + 8 * m4) = o;
    }
}

// ---------------------------------------------------------------- the same for ranks above 1024 (up to 4096)
// The query side of a rank this wide does not fit in LDS (3 limbs x R x 32 heads), and a wave's quarter of the value
// dims does not fit in registers, so both passes walk the latent in slabs of 1024 dims.  A workgroup owns up to NC
// chunks of 128 tokens.  Scores: for every slab the limbs of that slab are staged once and all the workgroup's chunks
// run against them, the integer dot products of a slab being added to a float score per (token, head).  Softmax: one
// maximum per head over all the workgroup's tokens (no running rescale), P kept in LDS as fp16.  Values: for every slab
// a wave accumulates its quarter of the slab's dims over all chunks and writes that piece of the partial result.
// The per-head scale of the integer query needs max |Q~| over the whole rank: k_shared_qmax computes it once per call.
__global__ __launch_bounds__(64) void k_shared_qmax(SharedParams p) {
  const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const float* q = p.qt + ((size_t)b * kSharedHeads + h) * p.R;
  float a = 0.f;
  for (int j0 = 0; j0 < p.R; j0 += 256) {                               // R is a multiple of 128: whole v4f pieces
    const int j = j0 + 4 * lane;
    if (j < p.R) {
      const v4f x = *(const v4f*)(q + j);
      a = fmaxf(a, fmaxf(fmaxf(fabsf(x[0]), fabsf(x[1])), fmaxf(fabsf(x[2]), fabsf(x[3]))));
    }
  }
  a = wave_max(a);
  if (lane == 0) p.qmax[b * kSharedHeads + h] = a;
}

constexpr int kBigSlab = 1024;            // latent dims per slab
constexpr int kBigChunks = 4;             // chunks of 128 tokens per workgroup, at most

__global__ __launch_bounds__(256) void k_shared_attn_big(SharedParams p) {
  constexpr int NC = kBigChunks;
  constexpr int NKS = kBigSlab / 32;      // 32-dim steps of a full slab
  constexpr int NKK = kBigSlab / 128;     // 32-dim value blocks one wave owns in a full slab
  extern __shared__ __align__(16) uint8_t sh_lds[];
  v4i* limbs = (v4i*)sh_lds;                                            // [3][NKS][64]
  float* cmax = (float*)(sh_lds + 3 * NKS * 1024);                      // [4][32]
  float* csum = cmax + 128;                                             // [4][32]
  float* ksc = csum + 128;                                              // [NC][4][32]
  _Float16* pt = (_Float16*)(ksc + NC * 128);                           // [NC][4 token blocks][32 heads][40]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, g2 = lane >> 5;
  const int split = blockIdx.x, b = blockIdx.y;
  const int R = p.R;
  const int n_b = min(max(p.seq_lens[b], 0), p.t_cap);
  const int n_chunks = (n_b + kSharedChunk - 1) / kSharedChunk;
  const int c0 = split * p.per, c1 = min(c0 + p.per, n_chunks);        // per <= NC by the launch's choice of splits
  const size_t part = (size_t)b * p.S + split;
  if (c0 >= c1) {                                                       // nothing for this split: the merge skips it
    if (tid < kSharedHeads) { p.pm[part * kSharedHeads + tid] = -INFINITY; p.pl[part * kSharedHeads + tid] = 0.f; }
    return;
  }
  const uint8_t* kplane = p.k_codes + (size_t)b * p.t_cap * R;
  const uint8_t* vplane = p.v_codes + (size_t)b * p.t_cap * R;
  const uint16_t* kmeta = p.k_scale + (size_t)b * p.t_cap;
  const uint16_t* vmeta = p.v_scale + (size_t)b * p.t_cap;
  const float hm = p.qmax[b * kSharedHeads + n];
  const float delta = hm > 0.f ? hm / kLimbRange : 1.0f;                // value of one unit of head n's integer query
  const float inv_delta = 1.0f / delta;
  const int n_slabs = (R + kBigSlab - 1) / kBigSlab;

  // K scales of this wave's 32 tokens of every chunk
#pragma unroll
  for (int c = 0; c < NC; c++)
    if (g2 == 0) ksc[(c * 4 + wave) * 32 + n] = c0 + c < c1 ? f16_bits_to_f32(kmeta[(c0 + c) * kSharedChunk + 32 * wave + n]) : 0.f;

  // ---- scores: sacc[c][v] = sum over the rank of (integer query of head n) . (codes of token row(v) of chunk c)
  float sacc[NC][16];
#pragma unroll
  for (int c = 0; c < NC; c++)
#pragma unroll
    for (int v = 0; v < 16; v++) sacc[c][v] = 0.f;
  const float* qrow = p.qt + ((size_t)b * kSharedHeads + n) * R + 16 * g2;
  for (int sl = 0; sl < n_slabs; sl++) {
    const int d0 = sl * kBigSlab;
    const int nks = min(kBigSlab, R - d0) >> 5;                         // a multiple of 4
    __syncthreads();                                                    // the previous slab's limbs are no longer read
    // this wave converts steps wave, wave + 4, ...: lane (n, g2) of step ks holds dims d0 + 32 ks + 16 g2 .. + 15
#pragma unroll
    for (int i0 = 0; i0 < NKS / 4; i0 += 4) {
      v4f xq[4][4];
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int ks = min(wave + 4 * (i0 + i), nks - 1);               // clamped: surplus steps are not stored
#pragma unroll
        for (int i4 = 0; i4 < 4; i4++) xq[i][i4] = *(const v4f*)(qrow + d0 + 32 * ks + 4 * i4);
      }
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int ks = wave + 4 * (i0 + i);
        if (ks < nks) {                                                 // wave-uniform
          v4i l0, l1, l2;
#pragma unroll
          for (int i4 = 0; i4 < 4; i4++) {
            uint32_t w0 = 0, w1 = 0, w2 = 0;
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const int Q = (int)__builtin_rintf(xq[i][i4][e] * inv_delta);
              const int a0 = ((Q + 64) & 127) - 64, Q1 = (Q - a0) >> 7;   // Q = a0 + 128 Q1 exactly
              const int a1 = ((Q1 + 64) & 127) - 64, a2 = (Q1 - a1) >> 7;
              w0 |= ((uint32_t)a0 & 0xFFu) << (8 * e);
              w1 |= ((uint32_t)a1 & 0xFFu) << (8 * e);
              w2 |= ((uint32_t)a2 & 0xFFu) << (8 * e);
            }
            l0[i4] = (int)w0; l1[i4] = (int)w1; l2[i4] = (int)w2;
          }
          limbs[(0 * NKS + ks) * 64 + lane] = l0;
          limbs[(1 * NKS + ks) * 64 + lane] = l1;
          limbs[(2 * NKS + ks) * 64 + lane] = l2;
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NC; c++) {
      if (c0 + c < c1) {                                                // workgroup-uniform
        const int t0 = (c0 + c) * kSharedChunk + 32 * wave;
        const uint8_t* kp = kplane + (size_t)(t0 >> 5) * (32 * (size_t)R) + (size_t)(d0 >> 5) * 1024 + (size_t)lane * 16;
        v16i a0, a1, a2;
#pragma unroll
        for (int v = 0; v < 16; v++) { a0[v] = 0; a1[v] = 0; a2[v] = 0; }
#pragma unroll
        for (int h0 = 0; h0 < NKS; h0 += 16) {
          if (h0 < nks) {                                               // nks is a multiple of 4, not of 16: see below
            v4i ka[16];
#pragma unroll
            for (int k = 0; k < 16; k++)
              ka[k] = __builtin_nontemporal_load((const v4i*)(kp + (size_t)min(h0 + k, nks - 1) * 1024));   // clamped, masked below
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 16; k++) {
              if (h0 + k < nks) {
                a0 = mfma_i8(ka[k], limbs[(0 * NKS + h0 + k) * 64 + lane], a0);
                a1 = mfma_i8(ka[k], limbs[(1 * NKS + h0 + k) * 64 + lane], a1);
                a2 = mfma_i8(ka[k], limbs[(2 * NKS + h0 + k) * 64 + lane], a2);
              }
              if ((k & 3) == 3) __builtin_amdgcn_sched_barrier(0);      // keeps the limb reads from piling up in registers
            }
          }
        }
#pragma unroll
        for (int v = 0; v < 16; v++) sacc[c][v] += fmaf(16384.f, (float)a2[v], fmaf(128.f, (float)a1[v], (float)a0[v]));
      }
    }
  }

  // ---- softmax over the workgroup's tokens: one maximum per head
  float bmax = -INFINITY;
#pragma unroll
  for (int c = 0; c < NC; c++) {
    const int t0 = (c0 + c) * kSharedChunk + 32 * wave;
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      const v4f k4 = *(const v4f*)&ksc[(c * 4 + wave) * 32 + 8 * m4 + 4 * g2];
#pragma unroll
      for (int jj = 0; jj < 4; jj++) {
        const int v = 4 * m4 + jj;
        const float sv = sacc[c][v] * delta * k4[jj];
        sacc[c][v] = (c0 + c < c1 && t0 + 8 * m4 + 4 * g2 + jj < n_b) ? sv : -INFINITY;   // rows past the sequence's end
        bmax = fmaxf(bmax, sacc[c][v]);
      }
    }
  }
  bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
  if (g2 == 0) cmax[wave * 32 + n] = bmax;
  __syncthreads();
  const float m_all = fmaxf(fmaxf(cmax[n], cmax[32 + n]), fmaxf(cmax[64 + n], cmax[96 + n]));   // finite: chunk c0 has a row
  float psum = 0.f;
#pragma unroll
  for (int c = 0; c < NC; c++) {
    _Float16* ptw = pt + ((c * 4 + wave) * 32 + n) * 40;
#pragma unroll
    for (int m4 = 0; m4 < 4; m4++) {
      v4f p4;
#pragma unroll
      for (int jj = 0; jj < 4; jj++) {
        const float sv = sacc[c][4 * m4 + jj];
        p4[jj] = sv == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sv - m_all);
        psum += p4[jj];
      }
      *(v2i*)&ptw[8 * m4 + 4 * g2] = __builtin_bit_cast(v2i, __builtin_convertvector(p4, v4f16));
    }
  }
  psum += __shfl_xor(psum, 32);
  if (g2 == 0) csum[wave * 32 + n] = psum;
  __syncthreads();
  if (wave == 0 && g2 == 0) {
    p.pm[part * kSharedHeads + n] = m_all;
    p.pl[part * kSharedHeads + n] = (csum[n] + csum[32 + n]) + (csum[64 + n] + csum[96 + n]);
  }

  // ---- values: slab by slab, this wave's quarter of the slab's dims over all chunks
  for (int sl = 0; sl < n_slabs; sl++) {
    const int d0 = sl * kBigSlab;
    const int nkk = min(kBigSlab, R - d0) >> 7;                         // 32-dim blocks per wave in this slab (1..8)
    const int blk0 = (d0 >> 5) + wave * nkk;                            // first 32-dim block of this wave
    v16f U[NKK];
#pragma unroll
    for (int kk = 0; kk < NKK; kk++)
#pragma unroll
      for (int v = 0; v < 16; v++) U[kk][v] = 0.f;
#pragma unroll
    for (int c = 0; c < NC; c++) {
      if (c0 + c < c1) {
        const int cbase = (c0 + c) * kSharedChunk;
        // all of the chunk's blocks of this slab are requested at once
        v4i vc[4][NKK], vsr[4][2];
#pragma unroll
        for (int tw = 0; tw < 4; tw++) {
          const int tv = min(cbase + 32 * tw, (n_b - 1) & ~31);         // (a block past the end: the last one again, unused)
          const uint8_t* vp = vplane + (size_t)(tv >> 5) * (32 * (size_t)R) + (size_t)blk0 * 1024 + (size_t)lane * 16;
#pragma unroll
          for (int kk = 0; kk < NKK; kk++) vc[tw][kk] = __builtin_nontemporal_load((const v4i*)(vp + (size_t)min(kk, nkk - 1) * 1024));
          vsr[tw][0] = *(const v4i*)(vmeta + tv + 16 * g2);
          vsr[tw][1] = *(const v4i*)(vmeta + tv + 16 * g2 + 8);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tw = 0; tw < 4; tw++) {
          const int tv = cbase + 32 * tw;
          if (tv < n_b) {
            v8f16 sv8[2] = {__builtin_bit_cast(v8f16, vsr[tw][0]), __builtin_bit_cast(v8f16, vsr[tw][1])};
            if (tv + 32 > n_b) {      // rows never written may hold any scale: they contribute 0
#pragma unroll
              for (int s2 = 0; s2 < 2; s2++)
#pragma unroll
                for (int e = 0; e < 8; e++)
                  if (tv + 16 * g2 + 8 * s2 + e >= n_b) sv8[s2][e] = (_Float16)0;
            }
            const v8f16 bp0 = *(const v8f16*)&pt[((c * 4 + tw) * 32 + n) * 40 + 16 * g2];
            const v8f16 bp1 = *(const v8f16*)&pt[((c * 4 + tw) * 32 + n) * 40 + 16 * g2 + 8];
#pragma unroll
            for (int kk = 0; kk < NKK; kk++) {
              if (kk < nkk) {                                           // workgroup-uniform
                U[kk] = mfma_f16(codes_f16(vc[tw][kk][0], vc[tw][kk][1]) * sv8[0], bp0, U[kk]);
                U[kk] = mfma_f16(codes_f16(vc[tw][kk][2], vc[tw][kk][3]) * sv8[1], bp1, U[kk]);
              }
            }
          }
        }
      }
    }
    float* pu = p.pu + (part * kSharedHeads + n) * R + (size_t)blk0 * 32 + 4 * g2;
#pragma unroll
    for (int kk = 0; kk < NKK; kk++) {
      if (kk < nkk) {
#pragma unroll
        for (int m4 = 0; m4 < 4; m4++) {
          v4f o;
#pragma unroll
          for (int jj = 0; jj < 4; jj++) o[jj] = U[kk][4 * m4 + jj];
          *(v4f*)(pu + 32 * kk + 8 * m4) = o;
        }
      }
    }
  }
}

// ---------------------------------------------------------------- merge of the splits and o_h = B_Vh^T u_h
// One workgroup per (head, kOutSeqs sequences).  (4 sequences per workgroup read B_Vh a quarter as often but leave
// three quarters of the CUs without a workgroup: measured 1.6 x slower at 16 sequences.)
constexpr int kOutSeqs = 1;
__global__ __launch_bounds__(256) void k_shared_out(SharedParams p) {
  extern __shared__ __align__(16) uint8_t so_lds[];
  float* wn = (float*)so_lds;                                           // [4][32 splits]: weight of a split / total sum
  float* uT = wn + kOutSeqs * 32;                                       // [R][kOutSeqs]
  float* red = uT + (size_t)p.R * kOutSeqs;                             // [16 slices][kOutSeqs][128 channels]
  const int tid = threadIdx.x, h = blockIdx.x, b0 = blockIdx.y * kOutSeqs;
  if ((tid >> 6) < kOutSeqs) {                                          // wave bi: lane s holds split s of sequence b0 + bi
    const int bi = tid >> 6, sidx = tid & 63, b = b0 + bi;
    const bool on = b < p.B && sidx < p.S;
    const float m = on ? p.pm[((size_t)b * p.S + sidx) * kSharedHeads + h] : -INFINITY;
    const float l = on ? p.pl[((size_t)b * p.S + sidx) * kSharedHeads + h] : 0.f;
    float M = m;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    const float w = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - M);
    float L = w * l;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) L += __shfl_xor(L, o);
    if (sidx < 32) wn[bi * 32 + sidx] = L > 0.f ? w / L : 0.f;
  }
  __syncthreads();
  for (int j = tid; j < p.R; j += 256)
#pragma unroll
    for (int bi = 0; bi < kOutSeqs; bi++) {
      float u = 0.f;
      if (b0 + bi < p.B) {
        const float* src = p.pu + (((size_t)(b0 + bi) * p.S) * kSharedHeads + h) * p.R + j;
        for (int s0 = 0; s0 < p.S; s0 += 16) {                          // 16 loads in flight (each trip of this loop is a
          float x[16];                                                  // memory round trip); a split that wrote nothing has
#pragma unroll                                                          // weight 0 and its (unwritten) values are dropped
          for (int i = 0; i < 16; i++) x[i] = src[(size_t)min(s0 + i, p.S - 1) * kSharedHeads * p.R];
#pragma unroll
          for (int i = 0; i < 16; i++) {
            const float w = s0 + i < p.S ? wn[bi * 32 + s0 + i] : 0.f;
            u += w != 0.f ? w * x[i] : 0.f;
          }
        }
      }
      uT[j * kOutSeqs + bi] = u;
    }
  __syncthreads();
  // thread (c8, js): output channels 8 c8 .. + 7 (one 16-byte load per row of B_Vh) over slice js of the R dims
  const int c8 = tid & 15, js = tid >> 4;
  float acc[kOutSeqs][8];
#pragma unroll
  for (int bi = 0; bi < kOutSeqs; bi++)
#pragma unroll
    for (int e = 0; e < 8; e++) acc[bi][e] = 0.f;
  if (8 * c8 < p.d) {
    const int jn = p.R >> 4;                                            // rows per slice: a multiple of 16
    const uint16_t* bv = p.BV + ((size_t)h * p.R + (size_t)js * jn) * p.d + 8 * c8;
    for (int j0 = 0; j0 < jn; j0 += 8) {                                // 8 loads in flight
      v4i w[8];
#pragma unroll
      for (int i = 0; i < 8; i++) w[i] = *(const v4i*)(bv + (size_t)(j0 + i) * p.d);
#pragma unroll
      for (int i = 0; i < 8; i++)
#pragma unroll
        for (int bi = 0; bi < kOutSeqs; bi++) {
          const float u = uT[(js * jn + j0 + i) * kOutSeqs + bi];
#pragma unroll
          for (int e2 = 0; e2 < 4; e2++) {
            acc[bi][2 * e2] = fmaf(u, __uint_as_float((uint32_t)w[i][e2] << 16), acc[bi][2 * e2]);
            acc[bi][2 * e2 + 1] = fmaf(u, __uint_as_float((uint32_t)w[i][e2] & 0xFFFF0000u), acc[bi][2 * e2 + 1]);
          }
        }
    }
#pragma unroll
    for (int bi = 0; bi < kOutSeqs; bi++)
#pragma unroll
      for (int e = 0; e < 8; e++) red[(js * kOutSeqs + bi) * 128 + 8 * c8 + e] = acc[bi][e];
  }
  __syncthreads();
  for (int i = tid; i < kOutSeqs * p.d; i += 256) {
    const int bi = i / p.d, c = i % p.d;
    if (b0 + bi < p.B) {
      float o = 0.f;
#pragma unroll
      for (int q = 0; q < 16; q++) o += red[(q * kOutSeqs + bi) * 128 + c];
      p.out[((size_t)(b0 + bi) * kSharedHeads + h) * p.d + c] = o;
    }
  }
}

int shared_splits(int batch, int t_cap, int rank) {
  int s = (256 + batch - 1) / batch;
  const int chunks = (t_cap + kSharedChunk - 1) / kSharedChunk;
  if (s > chunks) s = chunks;
  // ranks above 1024: a workgroup holds the scores of at most kBigChunks chunks
  if (rank > 1024 && s < (chunks + kBigChunks - 1) / kBigChunks) s = (chunks + kBigChunks - 1) / kBigChunks;
  if (s > 32) s = 32;
  return s < 1 ? 1 : s;
}

}  // namespace

size_t wsvd_shared_ws_bytes(int batch, int rank, int t_cap) {
  const size_t S = (size_t)shared_splits(batch, t_cap, rank);
  const size_t floats = (size_t)batch * kSharedHeads * rank + 2 * (size_t)batch * S * kSharedHeads + (size_t)batch * S * kSharedHeads * rank +
                        (size_t)batch * kSharedHeads;
  return floats * sizeof(float);
}

hipError_t wsvd_launch_attn_shared(int batch, int d_head, int rank, int t_cap, float sm_scale, const void* q, const void* B_K,
                                   const void* B_V, const void* k_codes, const void* v_codes, const void* k_scale,
                                   const void* v_scale, const int* seq_lens, void* workspace, void* out, hipStream_t s) {
  SharedParams p;
  p.q = (const uint16_t*)q; p.BK = (const uint16_t*)B_K; p.BV = (const uint16_t*)B_V;
  p.k_codes = (const uint8_t*)k_codes; p.v_codes = (const uint8_t*)v_codes;
  p.k_scale = (const uint16_t*)k_scale; p.v_scale = (const uint16_t*)v_scale;
  p.seq_lens = seq_lens;
  p.B = batch; p.d = d_head; p.R = rank; p.t_cap = t_cap; p.S = shared_splits(batch, t_cap, rank);
  const int chunks_cap = (t_cap + kSharedChunk - 1) / kSharedChunk;
  p.per = (chunks_cap + p.S - 1) / p.S;
  if (rank > 1024 && (p.per > kBigChunks || rank % 128 != 0 || rank > 4096)) return hipErrorNotSupported;
  p.c_scale = sm_scale * 1.4426950408889634f;
  p.qt = (float*)workspace;
  p.pm = p.qt + (size_t)batch * kSharedHeads * rank;
  p.pl = p.pm + (size_t)batch * p.S * kSharedHeads;
  p.pu = p.pl + (size_t)batch * p.S * kSharedHeads;
  p.qmax = p.pu + (size_t)batch * p.S * kSharedHeads * rank;
  p.out = (float*)out;

  hipLaunchKernelGGL(k_shared_absorb, dim3((unsigned)(rank / 32), kSharedHeads), dim3(64), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  const size_t lds_out = (size_t)(kOutSeqs * 32 + rank * kOutSeqs + 16 * kOutSeqs * 128) * sizeof(float);
  static bool raised_out = false;                                       // up to 99 KB at rank 4096
  if (!raised_out) {
    e = hipFuncSetAttribute((const void*)k_shared_out, hipFuncAttributeMaxDynamicSharedMemorySize, (int)((128 + 4096 * kOutSeqs + 16 * kOutSeqs * 128) * sizeof(float)));
    if (e != hipSuccess) return e;
    raised_out = true;
  }
  if (rank > 1024) {
    hipLaunchKernelGGL(k_shared_qmax, dim3(kSharedHeads, (unsigned)batch), dim3(64), 0, s, p);
    const size_t lds_big = (size_t)3 * (kBigSlab / 32) * 1024 + (size_t)(2 + kBigChunks) * 128 * sizeof(float) +
                           (size_t)kBigChunks * 4 * 32 * 40 * sizeof(_Float16);
    static bool raised_big = false;
    if (!raised_big) {
      e = hipFuncSetAttribute((const void*)k_shared_attn_big, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_big);
      if (e != hipSuccess) return e;
      raised_big = true;
    }
    hipLaunchKernelGGL(k_shared_attn_big, dim3((unsigned)p.S, (unsigned)batch), dim3(256), lds_big, s, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_shared_out, dim3(kSharedHeads, (unsigned)((batch + kOutSeqs - 1) / kOutSeqs)), dim3(256), lds_out, s, p);
    return hipGetLastError();
  }
  const size_t lds_attn = (size_t)3 * (rank / 32) * 1024 + 4 * 128 * sizeof(float) + 4 * 32 * 40 * sizeof(_Float16);
  const void* fn = rank == 256 ? (const void*)k_shared_attn<256> : rank == 512 ? (const void*)k_shared_attn<512>
                                                                                 : (const void*)k_shared_attn<1024>;
  static bool raised[3] = {false, false, false};                        // the kernels' limit of dynamic LDS, raised once
  const int ri = rank == 256 ? 0 : rank == 512 ? 1 : 2;
  if (!raised[ri]) {
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_attn);
    if (e != hipSuccess) return e;
    raised[ri] = true;
  }
  dim3 grid((unsigned)p.S, (unsigned)batch);
  if (rank == 256) hipLaunchKernelGGL((k_shared_attn<256>), grid, dim3(256), lds_attn, s, p);
  else if (rank == 512) hipLaunchKernelGGL((k_shared_attn<512>), grid, dim3(256), lds_attn, s, p);
  else if (rank == 1024) hipLaunchKernelGGL((k_shared_attn<1024>), grid, dim3(256), lds_attn, s, p);
  else return hipErrorNotSupported;
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  hipLaunchKernelGGL(k_shared_out, dim3(kSharedHeads, (unsigned)((batch + kOutSeqs - 1) / kOutSeqs)), dim3(256), lds_out, s, p);
  return hipGetLastError();
}
