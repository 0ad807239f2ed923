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

// ---------------------------------------------------------------- MFMA path: one finishing workgroup per unit
// A unit = (plane, kv head, group of up to SB sequences).  Its contraction over d_model is cut into one LARGE share,
// taken by the unit's finishing workgroup, and NP small ones, taken by helper workgroups (NP = 2: half of d_model, and
// a quarter each; NP = 0: everything in one workgroup).  A helper sums its share and PUSHES the partial tile to the
// finisher as 8-byte words {value, tag} written through to memory; the finisher, busy with twice as much of the factor
// stream, asks for those words before it needs them and finds them valid when its own sum is done, adds them in
// helper order (so the result does not depend on timing), quantises, stores the rows and clears the words again.
// Compared with equal slices merged by "last arriver sums": no ticket, no wait for store acknowledgements, no read-back
// after the last arrival: three dependent memory round trips less on the launch's critical path, while 3 * 2 * Hkv
// workgroups still pull the factor stream instead of 2 * Hkv (a CU sustains only about 70 GB/s of such loads, so one
// workgroup per unit spends 5 us fetching its 384 KB).
// Helpers have the lower workgroup ids of their unit and never wait, so they are dispatched first and always finish;
// the finisher's wait is bounded all the same (WSVD_E_HIP in the status word if a word never arrives).
// Waves split the workgroup's share of d_model; a wave keeps the factor operands of its k-steps in registers
// (requested in two batches around the staging of the hidden states, which all waves copy into LDS with coalesced
// loads); partial tiles meet in LDS (in the hidden states' place) and are summed in wave order.
constexpr uint32_t kLLTag = 0x4C4C5701u;      // marks a pushed word as written by the running launch's helper

// DEFER (the decode step's projection launch): NP equal slices of d_model per (plane, kv head), no finisher and no
// hand-off inside the launch: every workgroup leaves its partial sums in p.defer_out, workgroup 0 of each group of
// sequences advances the lengths and marks the rows as pending; the attention launch that follows sums the slices in
// slice order, quantises and stores the rows (the kernel boundary is the hand-off).
template <int R, int NT, bool DEFER = false>
__global__ __launch_bounds__(NT) void k_append_split(AppendParams p, int SB, int xs_stride /* elements */, int NP,
                                                     unsigned long long* ll /* [units][groups][NP][SB * R] */) {
  extern __shared__ __align__(16) uint8_t app_lds[];
  __shared__ int n_loc[32];
  __shared__ int flag_sh;
  constexpr int RTC = (R + 31) / 32;          // 32-channel row tiles (R = 16 uses half a tile)
  constexpr int KB = 8;                       // k-steps (of 16 model dims) per batch of factor loads
  uint16_t* xs = (uint16_t*)app_lds;                            // [SB][xs_stride] hidden states (bf16)
  float (*red)[R + 1] = (float (*)[R + 1])app_lds;              // [NW * SB][R + 1] partial tiles, later [SB][R + 1] rows
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NW = blockDim.x >> 6;
  const int n_roles = DEFER ? NP : NP + 1;
  const int unit = (int)blockIdx.x / n_roles, role = (int)blockIdx.x % n_roles;     // role < NP: helper, NP: finisher
  const bool finisher = !DEFER && role == NP;
  const int pl = unit / p.Hkv, kv = unit % p.Hkv;
  const int b0 = (int)blockIdx.y * SB, nb = min(SB, p.B - b0);
  const int col = lane & 31, g = lane >> 5;
  [[maybe_unused]] const int tl_wg = (int)(blockIdx.y * gridDim.x + blockIdx.x);
  WSVD_STAMP(p.timeline, tl_wg, wave, 0);
  // the lengths first: nothing depends on them until the rows are stored
  const int nreg = finisher ? append_target_row(p, b0 + min(tid, nb - 1)) : 0;
  // ... and, for the finisher that will turn out to be the last one, the lengths it advances on its way out: asked for
  // now, they cost nothing then (nobody writes them before that)
  int n_bump = (finisher && !p.fused) ? p.seq_lens[p.one_seq >= 0 ? p.one_seq : min(tid, p.B - 1)] : 0;
  if (DEFER && blockIdx.x == 0) n_bump = p.seq_lens[b0 + min(tid, nb - 1)];
  const uint16_t* Ap = (const uint16_t*)p.A[pl];
  const uint16_t* xp = (const uint16_t*)p.x;
  // ---- this workgroup's share of the k-steps (16 model dims each), then this wave's share of that
  const int nks = p.E >> 4;
  const int nks_fin = DEFER ? 0 : NP ? (nks + 1) / 2 : nks;     // the finisher's share comes first
  const int per_helper = NP ? (nks - nks_fin + NP - 1) / NP : 0;
  const int wg_k0 = finisher ? 0 : min(nks, nks_fin + role * per_helper);
  const int wg_k1 = finisher ? nks_fin : min(nks, wg_k0 + per_helper);
  const int per_wave = (wg_k1 - wg_k0 + NW - 1) / NW;
  const int ks0 = min(wg_k1, wg_k0 + wave * per_wave), ks1 = min(wg_k1, ks0 + per_wave);
  unsigned long long* ll_unit = ll + ((size_t)(unit * gridDim.y + blockIdx.y) * (NP ? NP : 1)) * (size_t)(SB * R);
  v8bf aop[2][RTC][KB];
  // Only the k-steps of the wave's own part are requested (wave-uniform predicate): the CU's address pipeline moves
  // 64 bytes per clock, and with 16 waves asking for everything at once every surplus request delays the useful ones.
  auto load_a = [&](int buf, int k0) {
#pragma unroll
    for (int k = 0; k < KB; k++) {
      if (k0 + k < ks1) {
#pragma unroll
        for (int rt = 0; rt < RTC; rt++)
          aop[buf][rt][k] = *(const v8bf*)(Ap + (((size_t)(kv * RTC + rt) * (size_t)nks + (size_t)(k0 + k)) * 64 + lane) * 8);
      }
    }
  };
  // ---- hidden states of the share -> LDS: whole 16-byte pieces, four per thread and trip in flight (wave-uniform
  // predicate per piece); the factor batches go out between the first trip's requests and its LDS writes, so that a
  // wave's first 16 k-steps cost one round trip
  const int ppr = (wg_k1 - wg_k0) * 2;                          // 16-byte pieces per row
  bool first = true;
  for (int i0 = 0; i0 < nb * ppr || first; i0 += 4 * (int)blockDim.x) {
    v4i piece[4];
#pragma unroll
    for (int it = 0; it < 4; it++) {
      if (i0 + it * (int)blockDim.x + (wave << 6) < nb * ppr) {  // some lane of this wave has a piece
        const int i = min(i0 + it * (int)blockDim.x + tid, nb * ppr - 1);
        piece[it] = *(const v4i*)(xp + (size_t)(b0 + i / ppr) * p.E + (size_t)wg_k0 * 16 + (size_t)(i % ppr) * 8);
      }
    }
    if (first) { load_a(0, ks0); load_a(1, ks0 + KB); first = false; WSVD_STAMP(p.timeline, tl_wg, wave, 1); }
#pragma unroll
    for (int it = 0; it < 4; it++) {
      const int i = i0 + it * (int)blockDim.x + tid;
      if (i < nb * ppr) *(v4i*)&xs[(size_t)(i / ppr) * xs_stride + (i % ppr) * 8] = piece[it];
    }
  }
  if (tid < 32) n_loc[tid] = nreg;
  __syncthreads();
  WSVD_STAMP(p.timeline, tl_wg, wave, 2);
  // every user of the old lengths draws a ticket once it holds them; whoever draws the last one advances them
  const int ticket = (tid == 0 && finisher && !p.fused) ? append_reader_ticket(p) : 0;
  v16f acc[RTC];
#pragma unroll
  for (int rt = 0; rt < RTC; rt++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[rt][v] = 0.f;
  const uint16_t* xrow = xs + (size_t)min(col, nb - 1) * xs_stride + g * 8;   // columns past the group repeat its last row
  auto mul = [&](int buf, int k0) {
#pragma unroll
    for (int k = 0; k < KB; k++)
      if (k0 + k < ks1) {                                       // wave-uniform
        const v8bf xo = *(const v8bf*)(xrow + (k0 + k - wg_k0) * 16);
#pragma unroll
        for (int rt = 0; rt < RTC; rt++) acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[buf][rt][k], xo, acc[rt], 0, 0, 0);
      }
  };
  for (int k0 = ks0; k0 < ks1; k0 += 2 * KB) {
    mul(0, k0);
    if (k0 + 2 * KB < ks1) load_a(0, k0 + 2 * KB);              // (wave-uniform; nothing is requested past the wave's part)
    mul(1, k0 + KB);
    if (k0 + 3 * KB < ks1) load_a(1, k0 + 3 * KB);
  }
  WSVD_STAMP(p.timeline, tl_wg, wave, 3);
  // the finisher asks for the helpers' words now, one (sequence, channel) element per thread and helper: whatever
  // has arrived by the time its own sum is done needs no second look
  constexpr int NPMAX = 2, EPT = (32 * R + NT - 1) / NT;         // helpers; elements per thread (SB <= 32)
  unsigned long long w[EPT][NPMAX];
  if (finisher && NP) {
#pragma unroll
    for (int e = 0; e < EPT; e++) {
      const int i = min(tid + e * (int)blockDim.x, SB * R - 1);
#pragma unroll
      for (int h = 0; h < NPMAX; h++)
        w[e][h] = __hip_atomic_load(ll_unit + (size_t)min(h, NP - 1) * (SB * R) + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();                                              // the hidden states are no longer read: their LDS is reused
#pragma unroll
  for (int rt = 0; rt < RTC; rt++)
#pragma unroll
    for (int v = 0; v < 16; v++) {
      // lane holds sequence column `col`, channel rows 8*(v/4) + 4*g + v%4
      const int ch = rt * 32 + 8 * (v / 4) + 4 * g + (v % 4);
      if (ch < R && col < nb) red[wave * SB + col][ch] = acc[rt][v];
    }
  __syncthreads();
  WSVD_STAMP(p.timeline, tl_wg, wave, 4);
  // sum over the waves in wave order, one thread per (sequence, channel); the result replaces wave 0's partial, which
  // only this thread reads
#pragma unroll
  for (int e = 0; e < EPT; e++) {
    const int i = tid + e * (int)blockDim.x;
    if (i < nb * R) {
      const int row = i / R, j = i % R;
      float c = 0.f;
      for (int k = 0; k < NW; k++) c += red[k * SB + row][j];
      if constexpr (DEFER) {
        p.defer_out[(((size_t)role * 2 + pl) * p.B + b0 + row) * ((size_t)p.Hkv * R) + (size_t)kv * R + j] = c;
      } else if (!finisher) {
        // push: value and tag in one 8-byte store, written through; nobody waits for it
        const unsigned long long word = ((unsigned long long)kLLTag << 32) | (unsigned long long)__float_as_uint(c);
        __hip_atomic_store(ll_unit + (size_t)role * (SB * R) + (size_t)row * R + j, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        if (NP) {
          unsigned long long* src = ll_unit + (size_t)row * R + j;
#pragma unroll
          for (int h = 0; h < NPMAX; h++) {
            if (h < NP) {
              unsigned long long v = w[e][h];
              int budget = 1 << 16;
              while ((uint32_t)(v >> 32) != kLLTag && budget > 0) {
                __builtin_amdgcn_s_sleep(1);
                v = __hip_atomic_load(src + (size_t)h * (SB * R), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                budget--;
              }
              if ((uint32_t)(v >> 32) != kLLTag) atomicExch(p.err_word, (int)WSVD_E_HIP);   // never seen; keeps the kernel finite
              c += __uint_as_float((uint32_t)v);
              // cleared for the next launch (a kernel boundary lies between); written through like the push itself
              __hip_atomic_store(src + (size_t)h * (SB * R), 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
          }
        }
        red[row][j] = c;
      }
    }
  }
  if constexpr (DEFER) {
    if (blockIdx.x == 0 && tid < nb) {
      const bool ok = n_bump >= 0 && n_bump < p.t_cap;
      if (ok) p.seq_lens[b0 + tid] = n_bump + 1;
      else atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
      p.pending[b0 + tid] = ok ? 1 : 0;
    }
    WSVD_STAMP(p.timeline, tl_wg, wave, 5);
    return;
  }
  if (!finisher) return;
  __syncthreads();
  WSVD_STAMP(p.timeline, tl_wg, wave, 5);
  append_store_rows<R>(p, pl, kv, b0, nb, red, n_loc - b0);
  WSVD_STAMP(p.timeline, tl_wg, wave, 6);
  if (p.fused) return;
  // ---- the lengths: advanced by the last finisher to have drawn a ticket (all others hold their copies by then)
  __syncthreads();
  if (tid == 0) {
    const int last = (ticket == (int)(gridDim.x / (NP + 1) * gridDim.y) - 1);
    if (last) __hip_atomic_store(p.tickets + 2 * p.Hkv, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    flag_sh = last;
  }
  __syncthreads();
  if (!flag_sh) return;
  if (p.one_seq >= 0) {
    if (tid == 0) {
      const int n0 = n_bump;
      if (n0 >= 0) p.seq_lens[p.one_seq] = min(n0 + p.B, p.t_cap);
      if (n0 < 0 || n0 + p.B > p.t_cap) atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
    }
    return;
  }
  for (int b = tid; b < p.B; b += blockDim.x) {
    const int n = b == tid ? n_bump : p.seq_lens[b];            // (more sequences than threads: the rest is read now)
    if (n >= 0 && n < p.t_cap) p.seq_lens[b] = n + 1;
    else atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
  }
}

// sequences per workgroup: 16, or 32 for larger batches (all 32 columns of the matrix-core tile: half as many passes over
// the factors), fewer when the finisher's share of their hidden-state rows does not fit LDS
// helpers per unit: two for model dims from 1024 (one when the batch needs more than one group of 32 sequences: the
// finisher and one helper per unit and group are then one workgroup per CU for up to 64 sequences of 32 kv heads, a
// single round), none below (the "append_helpers" option overrides)
static int append_split_np(const wsvd_layer_desc& d, int opt_helpers = -1) {
  if (opt_helpers >= 0) return d.d_model >= 1024 ? opt_helpers : 0;
  return d.d_model >= 1024 ? (d.batch > 32 ? 1 : 2) : 0;
}
static int append_split_sb(const wsvd_layer_desc& d) {
  const int share = append_split_np(d) ? (d.d_model / 16 + 1) / 2 * 16 : d.d_model;
  int sb = d.batch > 16 ? 32 : 16;
  while (sb > 1 && (size_t)sb * (share + 8) * 2 > (size_t)144 * 1024) sb >>= 1;
  return sb;
}
static bool append_split_ok(const wsvd_layer_desc& d) {
  const int share = append_split_np(d) ? (d.d_model / 16 + 1) / 2 * 16 : d.d_model;
  return (size_t)append_split_sb(d) * (share + 8) * 2 <= (size_t)144 * 1024 && d.d_model % 16 == 0;
}
// 8-byte words the helpers push per launch (the workspace's append area holds them)
size_t wsvd_append_ll_words(const wsvd_layer_desc& d) {
  const int sb = append_split_sb(d);
  return (size_t)2 * d.n_kv_heads * ((d.batch + sb - 1) / sb) * 2 * sb * d.rank;
}

template <int R, int NT>
static hipError_t launch_append_split(const AppendParams& p, const wsvd_layer_desc& d, int opt_helpers, unsigned long long* ll,
                                      hipStream_t s) {
  const int np = append_split_np(d, opt_helpers), sb = append_split_sb(d);
  const int share = np ? (d.d_model / 16 + 1) / 2 * 16 : d.d_model;
  const int stride = share + 8;                           // row stride = 4 dwords mod 32 banks: conflict-free operand reads
  const int groups = (d.batch + sb - 1) / sb;
  const int nw = NT / 64;
  size_t lds = (size_t)sb * stride * 2;
  const size_t red_bytes = (size_t)nw * sb * (R + 1) * 4;
  if (red_bytes > lds) lds = red_bytes;
  static bool raised = false;                             // one attribute per instantiation (the template makes it so)
  if (!raised) {
    hipError_t e = hipFuncSetAttribute((const void*)k_append_split<R, NT>, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e != hipSuccess) return e;
    raised = true;
  }
  dim3 grid((unsigned)(2 * d.n_kv_heads * (np + 1)), (unsigned)groups);
  hipLaunchKernelGGL((k_append_split<R, NT>), grid, dim3(NT), lds, s, p, sb, stride, np, ll);
  return hipGetLastError();
}

static bool append_mfma_path(const wsvd_layer_desc& d);
// The decode step's projection launch: `ns` equal d_model slices per (plane, kv head), partial sums to p.defer_out.
template <int R, int NT>
static hipError_t launch_append_project(const AppendParams& p, const wsvd_layer_desc& d, int ns, hipStream_t s) {
  const int nks = d.d_model / 16;
  const int share = (nks + ns - 1) / ns * 16;
  const int stride = share + 8;
  int sb = 16;
  while (sb > 1 && (size_t)sb * stride * 2 > (size_t)144 * 1024) sb >>= 1;
  const int groups = (d.batch + sb - 1) / sb;
  const int nw = NT / 64;
  size_t lds = (size_t)sb * stride * 2;
  const size_t red_bytes = (size_t)nw * sb * (R + 1) * 4;
  if (red_bytes > lds) lds = red_bytes;
  if (lds > (size_t)150 * 1024) return hipErrorInvalidValue;
  static bool raised = false;
  if (!raised) {
    hipError_t e = hipFuncSetAttribute((const void*)k_append_split<R, NT, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e != hipSuccess) return e;
    raised = true;
  }
  dim3 grid((unsigned)(2 * d.n_kv_heads * ns), (unsigned)groups);
  hipLaunchKernelGGL((k_append_split<R, NT, true>), grid, dim3(NT), lds, s, p, sb, stride, ns, (unsigned long long*)nullptr);
  return hipGetLastError();
}

// slices of the decode step's projection launch: about one workgroup per CU, at most 4, slices of whole k-steps
int wsvd_step_slices(const wsvd_ctx* ctx, const wsvd_layer_desc& d) {
  int ns = ctx->opt.step_slices > 0 ? ctx->opt.step_slices : ctx->n_cu / (2 * d.n_kv_heads);
  if (ns > 4) ns = 4;
  while (ns > 1 && d.d_model / 16 / ns < 4) ns--;
  return ns < 1 ? 1 : ns;
}
bool wsvd_step_deferred_ok(const wsvd_layer_desc& d) {
  return append_mfma_path(d) && d.latent_dtype == WSVD_I8 && (d.rank == 32 || d.rank == 64) &&
         d.n_q_heads / d.n_kv_heads <= 4 && d.d_model % 16 == 0 && d.batch <= kAppendMaxB;
}
// where the step's partial sums and its pending words live: inside the sliced kernels' partial area of the workspace
bool wsvd_step_partials(const wsvd_ctx* ctx, const wsvd_layer_desc& d, float** parts, int** pending, int* n_parts) {
  AppendParams p;
  wsvd_cache none = {};
  wsvd_append_params(ctx, d, nullptr, nullptr, nullptr, nullptr, none, p);
  const int ns = wsvd_step_slices(ctx, d);
  const size_t part_floats = (size_t)ns * 2 * d.batch * d.n_kv_heads * d.rank;
  if (part_floats > (size_t)2 * d.n_kv_heads * (d.d_model / 64) * d.batch * d.rank) return false;
  *parts = p.partials; *pending = (int*)(p.partials + part_floats); *n_parts = ns;
  return true;
}
hipError_t wsvd_launch_append_project(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* A_K,
                                      const void* A_V, const wsvd_cache& cache, float** parts, int** pending, int* n_parts,
                                      hipStream_t s) {
  AppendParams p;
  wsvd_append_params(ctx, d, x, nullptr, A_K, A_V, cache, p);
  int ns = 0;
  if (!wsvd_step_partials(ctx, d, parts, pending, &ns)) return hipErrorNotSupported;
  p.defer_out = *parts;
  p.pending = *pending;
  if (ctx->opt.timeline_kernel != 1) p.timeline = nullptr;    // (profiling build: by default a step's stamps are its attention launch's)
  *n_parts = ns;
  switch (d.rank) {
    case 32: return launch_append_project<32, 512>(p, d, ns, s);      // (8 waves: 6.7 us at config 3; 16: 6.9 us; 4: 7.4 us)
    case 64: return launch_append_project<64, 512>(p, d, ns, s);
    default: return hipErrorNotSupported;
  }
}

// d_model slices per (plane, kv head).
// One CU cannot pull more than a few tens of GB/s on its own, so the factor stream has to be spread over all of
// them: the MFMA path aims at about one workgroup per CU (256) and merges the slices through the ticket.
// The vector-ALU path keeps slices of at most 256 elements (its LDS staging size).
static bool append_mfma_path(const wsvd_layer_desc& d) { return d.factor_dtype == WSVD_BF16 && d.x_dtype == WSVD_BF16; }
int wsvd_append_esplits(const wsvd_ctx* ctx, const wsvd_layer_desc& d) {
  if (!append_mfma_path(d)) {
    int esl = kAppendMaxESL;
    while (esl > 64 && d.d_model % esl != 0) esl >>= 1;
    return d.d_model / esl;
  }
  const int units = d.d_model / 64;                              // slices are multiples of 64 elements
  int want = ctx->opt.append_mode > 0 ? ctx->opt.append_mode : 256 / (2 * d.n_kv_heads);
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
static size_t wsvd_append_pushed_floats(const wsvd_layer_desc& d) {
  return append_mfma_path(d) && append_split_ok(d) ? (2 * wsvd_append_ll_words(d) + 3) / 4 * 4 : 0;
}
size_t wsvd_append_partial_floats(const wsvd_layer_desc& d) {
  // the pushed words of the default kernel (which are zero between launches), then the sliced kernels' partial sums
  // (the most slices an option can ask for)
  // (+ one word per sequence behind the decode step's partial sums, which use this area too)
  const size_t sliced = (size_t)2 * d.n_kv_heads * (d.d_model / 64) * d.batch * d.rank + ((size_t)d.batch + 3) / 4 * 4;
  return wsvd_append_pushed_floats(d) + sliced;
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
  p.partials = (float*)((char*)ctx->ws + (size_t)kWsCounterInts * 4) + (wsvd_attn_partial_floats(d) + 3) / 4 * 4 + wsvd_append_pushed_floats(d);
  p.err_word = ctx->err_word;
  p.B = d.batch; p.E = d.d_model; p.Hkv = d.n_kv_heads; p.t_cap = d.t_cap;
  p.ES = wsvd_append_esplits(ctx, d); p.ESL = d.d_model / p.ES;
  p.x_dtype = d.x_dtype; p.factor_dtype = d.factor_dtype; p.latent_dtype = d.latent_dtype;
  p.one_seq = -1;
  p.timeline = ctx->timeline_bytes >= (size_t)4096 * kTimelineWaves * kTimelineSlots * sizeof(long long) ? ctx->timeline : nullptr;
}

// waves per workgroup of the MFMA path: each wave gets a multiple of 16 elements, at least 64; up to 16 waves
// (rank 64: 8, register budget)
int wsvd_append_mfma_waves(const wsvd_ctx* ctx, const wsvd_layer_desc& d) {
  const int esl = d.d_model / wsvd_append_esplits(ctx, d);
  int nw = d.rank == 64 ? 8 : 16;
  while (nw > 4 && ((esl / nw) % 16 != 0 || esl / nw < 64)) nw >>= 1;
  return nw;
}
bool wsvd_append_uses_mfma(const wsvd_layer_desc& d) { return append_mfma_path(d); }

hipError_t wsvd_launch_append(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale,
                              const void* A_K, const void* A_V, const wsvd_cache& cache, hipStream_t s, int one_seq,
                              const wsvd_paged_cache* paged) {
  if (paged && !(d.rank <= 64 && append_mfma_path(d) && ctx->opt.append_mode == 0 && append_split_ok(d) &&
                 (d.latent_dtype == WSVD_I8 || d.latent_dtype == WSVD_I4)))
    return hipErrorNotSupported;           // paged cache: quantised latents through the default kernel
  if (d.rank > 64) {
    // ranks 96 / 128 (int8 latents, bf16 hidden states and factors): the tiled projection with one token per sequence,
    // then its length update: two launches
    if (one_seq >= 0) return hipErrorNotSupported;
    return wsvd_launch_prefill_project(ctx, d, x, 1, -1, A_K, A_V, cache, s);
  }
  AppendParams p;
  wsvd_append_params(ctx, d, x, x_scale, A_K, A_V, cache, p);
  p.one_seq = one_seq;
  if (paged) { p.block_table = paged->block_table; p.page_rows = paged->page_rows; p.max_pages = paged->max_pages; p.n_pages = paged->n_pages; }
  if (d.d_model % 64 != 0 || d.batch > kAppendMaxB) return hipErrorInvalidValue;
  dim3 grid((unsigned)(p.ES * p.Hkv * 2));
  const bool f32 = d.factor_dtype == WSVD_F32;
  if (append_mfma_path(d) && ctx->opt.append_mode == 0 && append_split_ok(d)) {
    // the default ("append_mode" n > 0 asks for the kernel with n equal slices merged by the last arriver instead)
    unsigned long long* ll = (unsigned long long*)((char*)ctx->ws + (size_t)kWsCounterInts * 4 + (wsvd_attn_partial_floats(d) + 3) / 4 * 16);
    switch (d.rank) {
      case 16: return launch_append_split<16, 1024>(p, d, ctx->opt.append_helpers, ll, s);
      case 32: return launch_append_split<32, 1024>(p, d, ctx->opt.append_helpers, ll, s);
      case 64: return launch_append_split<64, 512>(p, d, ctx->opt.append_helpers, ll, s);
      default: return hipErrorInvalidValue;
    }
  }
  if (append_mfma_path(d)) {
    int nw = wsvd_append_mfma_waves(ctx, d);
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
