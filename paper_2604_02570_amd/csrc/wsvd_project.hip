// Cache build for a whole prompt (the projection of prefilling, Section 3.4): C = x A for all prompt tokens on the matrix
// cores, per-token int8 quantisation and stores in the decode layout.
#include "wsvd_dev.h"
#include "wsvd_internal.h"

namespace {

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
  int i4;                           // int4 latents (rank 32): asymmetric codes, two rows per value byte
  // paged cache only (else null): codes / meta are pools of n_pages pages, a page = page_rows rows of every kv head in the
  // layout of a contiguous plane; block_table [B][max_pages]
  const int* block_table;
  int page_rows, max_pages, n_pages;
};

// Where row t of (sequence, kv head) lives: its plane (row_bytes per row), its row inside that plane, the index of its
// metadata entry.  Paged: a table entry outside the pools is reported and the row is not stored (ok = false).
struct ProjRow { uint8_t* plane; size_t meta; int t; bool ok; };
WSVD_DEV ProjRow project_row(const ProjectParams& p, int pl, int seq, int kv, int t, int row_bytes) {
  ProjRow r;
  if (!p.block_table) {
    const size_t ph = (size_t)seq * p.Hkv + kv;
    r.plane = p.codes[pl] + ph * (size_t)p.t_cap * row_bytes; r.meta = ph * p.t_cap + t; r.t = t; r.ok = true;
    return r;
  }
  const int pg = min(max(t, 0) / p.page_rows, p.max_pages - 1);
  const int e = p.block_table[(size_t)seq * p.max_pages + pg];
  r.ok = e >= 0 && e < p.n_pages;
  if (!r.ok) atomicExch(p.err_word, (int)WSVD_E_SHAPE);
  const size_t slot = (size_t)(r.ok ? e : 0) * p.Hkv + kv;
  r.t = t - pg * p.page_rows;
  r.plane = p.codes[pl] + slot * (size_t)p.page_rows * row_bytes;
  r.meta = slot * p.page_rows + r.t;
  return r;
}

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
      const int tok = (tb * TT + tt) * 32 + n;                          // this lane's token of the prompt
      const int t = n0 + tok;                                           // and its cache row
      if constexpr (R == 32) {
        if (p.i4) {
          // int4 (rank 32: one channel tile per head): the rule of quantize_row_i4 on the 16 channels this lane holds
          // and the 16 of its partner half; K bytes pair dims (2 adjacent registers), V bytes pair rows t, t ^ 1 = this
          // lane and its neighbour (the caller guarantees an even start row, so row parity = lane parity)
          float lo = 0.f, hi = 0.f;
#pragma unroll
          for (int v = 0; v < 16; v++) { lo = fminf(lo, acc[h][tt][v]); hi = fmaxf(hi, acc[h][tt][v]); }
          lo = fminf(lo, __shfl_xor(lo, 32)); hi = fmaxf(hi, __shfl_xor(hi, 32));
          uint16_t sh = 0x3C00u;
          float z = 0.f;
          const bool flat = (hi == lo);
          if (!flat) sh = guard_scale_f16((hi - lo) / 15.0f);
          const float sc = f16_bits_to_f32(sh);
          if (!flat) z = fminf(fmaxf(__builtin_rintf(-lo / sc), 0.f), 15.f);
          const int zi = (int)z;
          bool on = tok < p.n_tok && n0 >= 0 && (n0 & 1) == 0 && t < p.t_cap;
          ProjRow pr = {p.codes[pl] + ph * (size_t)p.t_cap * 16, ph * p.t_cap + t, t, true};
          if (p.block_table && on) { pr = project_row(p, pl, seq, kv, t, 16); on = pr.ok; }
          uint8_t* plane4 = pr.plane;
          const int tr = pr.t;
#pragma unroll
          for (int m4 = 0; m4 < 4; m4++) {
            int q[4];
#pragma unroll
            for (int jj = 0; jj < 4; jj++) {
              const float v = fminf(fmaxf(__builtin_rintf(acc[h][tt][4 * m4 + jj] / sc), -64.f), 64.f);
              const int qq = (int)v + zi;
              q[jj] = qq < 0 ? 0 : (qq > 15 ? 15 : qq);
            }
            const int j0 = 8 * m4 + 4 * g2;                             // channels j0 .. j0 + 3
            if (pl == 0) {
              int nib;
              if (on) *(uint16_t*)(plane4 + i4_k_offset(tr, j0, &nib)) = (uint16_t)(q[0] | (q[1] << 4) | (q[2] << 8) | (q[3] << 12));
            } else {
#pragma unroll
              for (int jj = 0; jj < 4; jj++) {
                const int qn = __builtin_amdgcn_update_dpp(0, q[jj], kDppQuadSwap1, 0xF, 0xF, true);   // the neighbour row's code
                const bool nb_on = tok + 1 < p.n_tok && t + 1 < p.t_cap;
                int nib;
                if (on && (n & 1) == 0) plane4[i4_v_offset(tr, j0 + jj, &nib)] = (uint8_t)(q[jj] | ((nb_on ? qn : 0) << 4));
              }
            }
          }
          if (on && g2 == 0) *(uint32_t*)&p.meta[pl][pr.meta * 2] = (uint32_t)sh | ((uint32_t)f32_to_f16_bits_rne((float)zi) << 16);
          continue;
        }
      }
      float a = 0.f;
#pragma unroll
      for (int rt = 0; rt < RT; rt++)
#pragma unroll
        for (int v = 0; v < 16; v++) a = fmaxf(a, fabsf(acc[h * RT + rt][tt][v]));
      a = fmaxf(a, __shfl_xor(a, 32));
      uint16_t sh = 0x3C00u;
      if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
      const float sc = f16_bits_to_f32(sh);
      if (tok >= p.n_tok || n0 < 0 || t >= p.t_cap) continue;
      ProjRow pr = {plane, ph * p.t_cap + t, t, true};
      if (p.block_table) { pr = project_row(p, pl, seq, kv, t, R); if (!pr.ok) continue; }
      uint8_t* const pln = pr.plane;
      const int tr = pr.t;
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
          if (pl == 0) *(uint32_t*)(pln + i8_k_offset(tr, j0, R)) = pk;
          else {
#pragma unroll
            for (int jj = 0; jj < 4; jj++) pln[i8_v_offset(tr, j0 + jj, R)] = (uint8_t)q[jj];
          }
        }
      if (g2 == 0) p.meta[pl][pr.meta] = sh;
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

template <int R, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k_prefill_project_lds(ProjectParams p) {
  extern __shared__ __align__(16) uint8_t proj_lds[];
  constexpr int RT = R / 32, CT = 4, TT = 16 / WAVES;                   // 2 x (WAVES / 2) waves, each 4 x TT tiles
  constexpr int NT = 64 * WAVES, NLD = 2048 / NT;                       // threads; 16-byte pieces of A (and of x) per thread and chunk
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
  const uint8_t* asrc[NLD];
  const uint8_t* xbase = (const uint8_t*)p.x + (size_t)sq * p.n_tok * p.E * 2;
  uint32_t xoff[NLD];
  int xdst[NLD];
  const uint32_t aoff = (tid & 255) * 16;
#pragma unroll
  for (int j = 0; j < NLD; j++) {
    const int u = tid + NT * j;                                         // piece u: tile u / 256 of A, row u / 8 of x
    const int ct = min(cg * 8 + (u >> 8), tiles - 1);
    asrc[j] = (const uint8_t*)p.A[ct / tiles_plane] + (size_t)(ct % tiles_plane) * n_steps * 1024;
    const int row = u >> 3, sg = u & 7;
    const int tok = min(by * 256 + row, p.n_tok - 1);
    xoff[j] = (uint32_t)tok * (uint32_t)(p.E * 2) + sg * 16;            // the launcher keeps n_tok * E * 2 below 2^31
    xdst[j] = kProjABytes + row * kProjXRow + sg * 16;
  }
  v4u rg[2 * NLD];                                                      // the chunk on its way: NLD pieces of A, NLD of x
  auto fetch1 = [&](int j, int c) {
    c = min(c, n_chunks - 1);                     // (past the end: the last chunk again, written to the idle stage, never read)
    if (j < NLD) rg[j] = *(const v4u*)(asrc[j] + (size_t)c * 4096 + aoff);
    else rg[j] = *(const v4u*)(xbase + (size_t)c * (kProjKC * 2) + xoff[j - NLD]);
  };
  auto commit1 = [&](int j, int st) {
    uint8_t* base = proj_lds + st * kProjStage;
    if (j < NLD) *(v4u*)(base + (tid + NT * j) * 16) = rg[j];
    else *(v4u*)(base + xdst[j - NLD]) = rg[j];
  };
  v16f acc[CT][TT];
#pragma unroll
  for (int c = 0; c < CT; c++)
#pragma unroll
    for (int tt = 0; tt < TT; tt++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[c][tt][v] = 0.f;
  const int a_off = wc * 4 * 4096 + lane * 16;                          // + c * 4096 + ks * 1024
  const int x_off = kProjABytes + (wt * 32 * TT + n) * kProjXRow + g2 * 16; // + tt * 32 rows + ks * 32 bytes
#pragma unroll
  for (int j = 0; j < 2 * NLD; j++) fetch1(j, 0);
#pragma unroll
  for (int j = 0; j < 2 * NLD; j++) commit1(j, 0);
  __syncthreads();
  // One or two waves per SIMD: little else fills the issue slots a wave leaves empty, so the order of its instructions
  // is fixed by hand.  Per step of 16 model dims: the operand reads of the NEXT step, then 4 groups of TT products, each
  // followed, in the first two steps, by its share of the 16-byte requests of the next chunk and, in the last step, by
  // its share of the 16-byte writes of it to the idle stage: requests and writes trickle into the memory pipelines
  // between products instead of blocking the wave in a burst.
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
        if (ks < 2) {
#pragma unroll
          for (int j = 0; j < NLD / 4; j++) fetch1((NLD / 4) * (ks * 4 + cc) + j, c + 1);
        }
        if (ks == 3) {
#pragma unroll
          for (int j = 0; j < NLD / 2; j++) commit1((NLD / 2) * cc + j, (c + 1) & 1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
  }
  const int ct0 = (cg * 2 + wc) * CT, tb = by * (8 / TT) + wt;
  if (ct0 >= tiles || tb * 32 * TT >= p.n_tok) return;
  project_store<R, CT, TT>(p, acc, ct0, tb, seq, n0);
}

// after the projection: the lengths move on by the rows that fitted (one thread per sequence)
__global__ void k_prefill_bump(int* seq_lens, int seq0, int n_seq, int n_tok, int t_cap, int* err_word, int even_only) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_seq) return;
  const int n0 = seq_lens[seq0 + i];
  if (even_only && n0 >= 0 && (n0 & 1)) {      // int4: nothing was stored for a sequence that starts on an odd row
    atomicExch(err_word, (int)WSVD_E_SHAPE);
    return;
  }
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


hipError_t wsvd_launch_prefill_project(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, int n_tok, int seq,
                                       const void* A_K, const void* A_V, const wsvd_cache& cache, hipStream_t s,
                                       const wsvd_paged_cache* paged) {
  const bool i4 = d.latent_dtype == WSVD_I4 && d.rank == 32;
  if (paged && d.rank > 64) return hipErrorNotSupported;
  if ((d.latent_dtype != WSVD_I8 && !i4) || d.factor_dtype != WSVD_BF16 || d.x_dtype != WSVD_BF16) return hipErrorNotSupported;
  if (d.rank != 32 && d.rank != 64 && d.rank != 96 && d.rank != 128) return hipErrorNotSupported;
  if (d.d_model % 16 != 0 || n_tok < 1) return hipErrorInvalidValue;
  ProjectParams p;
  p.x = (const uint16_t*)x; p.A[0] = (const uint16_t*)A_K; p.A[1] = (const uint16_t*)A_V;
  p.codes[0] = (uint8_t*)cache.k_codes; p.codes[1] = (uint8_t*)cache.v_codes;
  p.meta[0] = (uint16_t*)cache.k_meta; p.meta[1] = (uint16_t*)cache.v_meta;
  p.seq_lens = cache.seq_lens; p.err_word = ctx->err_word;
  p.Hkv = d.n_kv_heads; p.E = d.d_model; p.t_cap = d.t_cap; p.n_tok = n_tok;
  p.n_cg = p.tg_seq = p.n_tg = 0;
  p.i4 = i4 ? 1 : 0;
  p.block_table = nullptr; p.page_rows = p.max_pages = p.n_pages = 0;
  if (paged) { p.block_table = paged->block_table; p.page_rows = paged->page_rows; p.max_pages = paged->max_pages; p.n_pages = paged->n_pages; }
  const int n_seq = seq < 0 ? d.batch : 1;
  p.seq0 = seq < 0 ? 0 : seq;
  // small problems: small wave tiles, so that there are enough waves; prompt-sized ones: the LDS-staged kernel
  // (option "project_shape": 1 = staged, 44 / 42 / 24 / 21 = variants of the direct kernel, for tuning and tests)
  const long long work = (long long)n_seq * n_tok * d.n_kv_heads * d.rank;
  const bool staged_ok = d.d_model % kProjKC == 0 && (long long)n_tok * d.d_model * 2 < (1LL << 31);
  int shape = ctx->opt.project_shape ? ctx->opt.project_shape : (work >= (1LL << 22) ? (staged_ok ? 1 : 44) : 21);
  if ((shape == 1 || shape == 2) && !staged_ok) shape = 44;
  if (i4 && (shape == 1 || shape == 2)) shape = 44;      // int4: the direct kernels (the staged one stores int8 rows only)
  if (d.rank > 64) {
    // ranks 96 / 128: a wave owns the 3 / 4 channel tiles of one head and 1 or 4 token tiles
    const bool big = work >= (1LL << 22);
    if (d.rank == 96) { if (big) launch_project<96, 3, 4, 4>(p, n_seq, s); else launch_project<96, 3, 1, 4>(p, n_seq, s); }
    else { if (big) launch_project<128, 4, 4, 4>(p, n_seq, s); else launch_project<128, 4, 1, 4>(p, n_seq, s); }
  } else if (shape == 1 || shape == 2) {
    const int tiles = 2 * p.Hkv * (d.rank / 32);
    p.n_cg = (tiles + 7) / 8; p.tg_seq = (n_tok + 255) / 256; p.n_tg = p.tg_seq * n_seq;
    dim3 grid((unsigned)(p.n_cg * p.n_tg));
    const size_t lds = 2 * (size_t)kProjStage;
    static bool raised[4] = {false, false, false, false};   // the kernels' limit of dynamic LDS, raised once
    const bool w8 = shape == 2;
    const void* fn = d.rank == 32 ? (w8 ? (const void*)k_prefill_project_lds<32, 8> : (const void*)k_prefill_project_lds<32, 4>)
                                  : (w8 ? (const void*)k_prefill_project_lds<64, 8> : (const void*)k_prefill_project_lds<64, 4>);
    const int fi = (d.rank == 64) * 2 + w8;
    if (!raised[fi]) {
      hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      raised[fi] = true;
    }
    if (d.rank == 32 && !w8) hipLaunchKernelGGL((k_prefill_project_lds<32, 4>), grid, dim3(256), lds, s, p);
    else if (d.rank == 32) hipLaunchKernelGGL((k_prefill_project_lds<32, 8>), grid, dim3(512), lds, s, p);
    else if (!w8) hipLaunchKernelGGL((k_prefill_project_lds<64, 4>), grid, dim3(256), lds, s, p);
    else hipLaunchKernelGGL((k_prefill_project_lds<64, 8>), grid, dim3(512), lds, s, p);
  } else if (d.rank == 32) {
    if (shape == 44) launch_project<32, 4, 4, 4>(p, n_seq, s);
    else if (shape == 42) launch_project<32, 4, 2, 4>(p, n_seq, s);
    else if (shape == 24) launch_project<32, 2, 4, 4>(p, n_seq, s);
    else launch_project<32, 2, 1, 4>(p, n_seq, s);
  } else {
    if (shape == 44) launch_project<64, 4, 4, 4>(p, n_seq, s);
    else if (shape == 42) launch_project<64, 4, 2, 4>(p, n_seq, s);
    else if (shape == 24) launch_project<64, 2, 4, 4>(p, n_seq, s);
    else launch_project<64, 2, 1, 4>(p, n_seq, s);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_prefill_bump, dim3((n_seq + 63) / 64), dim3(64), 0, s, cache.seq_lens, p.seq0, n_seq, n_tok, d.t_cap, ctx->err_word, p.i4);
  return hipGetLastError();
}
