// Decode attention over I8 / I4 latent caches on the gfx950 matrix cores.
//
// The cache planes are stored as MFMA operand images (layout in wsvd.h), so the 16 bytes a lane loads
// ARE its slice of the B operand of V_MFMA_I32_32X32X32_I8: no unpack for I8, two mask/shift pairs per
// dword for I4.  The float side of each product is carried as three 7-bit limbs:
//   * score pass:  q~ (B_K folded into the query) = delta * (h*2^14 + m*2^7 + l); rows of the A operand
//     are the limbs, columns of B are tokens, so D[limb][token] are exact int32 dot products;
//   * value pass:  w_t = p_t * scale_V[t] = omega * (h*2^14 + m*2^7 + l); A rows are the limbs over tokens
//     (transposed through LDS), B is the token-minor V block, D[limb][dim] accumulates exactly in int32
//     ACROSS tiles for as long as the softmax reference m and the weight unit omega stay put.
// A tile is 64 tokens: two 32-token blocks whose score MFMAs are chained into disjoint row groups so
// that lane L ends up with the scores of token L of the tile.
// The online softmax is lazy: the wave-wide max reduction, the rescale of the accumulators and the
// int32 -> float flush only run for tiles that raise the running max or overflow the weight unit
// (wave-uniform branches); the common tile costs a few dozen vector-ALU instructions.
// Operand / result register layouts used here were checked on hardware:
//   A: lane L holds row L%32, k = 16*(L/32)..+15;  B: lane L holds column L%32, same k;
//   D: lane L, register v holds row 8*(v/4) + 4*(L/32) + v%4, column L%32.
#include <type_traits>

#include "wsvd_attn_common.h"
#include "wsvd_append_body.h"
#include "wsvd_internal.h"

template <int R, bool I4>
struct TileRegs {
  // I8: k[kk][blk], v[jj][blk] with kk, jj < R/32 and blk < 2.  I4 (R == 32): k[0][0], v[0][0] hold 64 tokens.
  v4i k[R / 32][2];
  v4i v[R / 32][2];
  uint32_t kmeta, vmeta;   // I8: fp16 scale in the low half; I4: scale | zero point << 16
};

// A tile's loads come in two halves, in the order its data is needed: the key side (code blocks and metadata of
// the keys: all the score pass needs) and the value side (metadata first: the weights need the scales before the value
// pass needs the codes).  Loads return in issue order, so the score pass starts while the value side is still on
// its way.
template <int R, bool I4>
WSVD_DEV void load_tile_k(TileRegs<R, I4>& t, const uint8_t* kplane, const uint16_t* kmeta, int tile, int lane) {
  const uint32_t moff = (uint32_t)tile * 64u + (uint32_t)lane;
  if (I4) {
    t.k[0][0] = __builtin_nontemporal_load((const v4i*)(kplane + (uint32_t)tile * 1024u + (uint32_t)lane * 16u));
    t.kmeta = __builtin_nontemporal_load((const uint32_t*)kmeta + moff);
  } else {
    const uint32_t off = (uint32_t)tile * (uint32_t)(64 * R) + (uint32_t)lane * 16u;
#pragma unroll
    for (int blk = 0; blk < 2; blk++)
#pragma unroll
      for (int kk = 0; kk < R / 32; kk++)
        t.k[kk][blk] = __builtin_nontemporal_load((const v4i*)(kplane + off + (uint32_t)(blk * (32 * R) + kk * 1024)));
    t.kmeta = __builtin_nontemporal_load(kmeta + moff);
  }
}
template <int R, bool I4>
WSVD_DEV void load_tile_v(TileRegs<R, I4>& t, const uint8_t* vplane, const uint16_t* vmeta, int tile, int lane) {
  const uint32_t moff = (uint32_t)tile * 64u + (uint32_t)lane;
  if (I4) {
    t.vmeta = __builtin_nontemporal_load((const uint32_t*)vmeta + moff);
    t.v[0][0] = __builtin_nontemporal_load((const v4i*)(vplane + (uint32_t)tile * 1024u + (uint32_t)lane * 16u));
  } else {
    const uint32_t off = (uint32_t)tile * (uint32_t)(64 * R) + (uint32_t)lane * 16u;
    t.vmeta = __builtin_nontemporal_load(vmeta + moff);
#pragma unroll
    for (int blk = 0; blk < 2; blk++)
#pragma unroll
      for (int kk = 0; kk < R / 32; kk++)
        t.v[kk][blk] = __builtin_nontemporal_load((const v4i*)(vplane + off + (uint32_t)(blk * (32 * R) + kk * 1024)));
  }
}
// All offsets are 32-bit and relative to wave-uniform plane pointers, so the loads use the
// scalar-base + vector-offset addressing form (one address instruction per tile).
template <int R, bool I4>
WSVD_DEV void load_tile(TileRegs<R, I4>& t, const uint8_t* kplane, const uint8_t* vplane, const uint16_t* kmeta,
                        const uint16_t* vmeta, int tile, int lane) {
  load_tile_k<R, I4>(t, kplane, kmeta, tile, lane);
  load_tile_v<R, I4>(t, vplane, vmeta, tile, lane);
}

// The same tile through agent-scope loads (dword granularity): coherent with write-through stores made by other
// workgroups of the running launch.
WSVD_DEV v4i load16_coherent(const uint8_t* a) {
  v4i r;
#pragma unroll
  for (int i = 0; i < 4; i++) r[i] = __hip_atomic_load((const int*)a + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return r;
}
template <int R, bool I4>
WSVD_DEV void load_tile_coherent(TileRegs<R, I4>& t, const uint8_t* kplane, const uint8_t* vplane, const uint16_t* kmeta,
                                 const uint16_t* vmeta, int tile, int lane) {
  if (I4) {
    const uint32_t off = (uint32_t)tile * 1024u + (uint32_t)lane * 16u;
    t.k[0][0] = load16_coherent(kplane + off);
    t.v[0][0] = load16_coherent(vplane + off);
    const uint32_t moff = (uint32_t)tile * 64u + (uint32_t)lane;
    t.kmeta = __hip_atomic_load((const uint32_t*)kmeta + moff, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    t.vmeta = __hip_atomic_load((const uint32_t*)vmeta + moff, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    const uint32_t off = (uint32_t)tile * (uint32_t)(64 * R) + (uint32_t)lane * 16u;
#pragma unroll
    for (int blk = 0; blk < 2; blk++)
#pragma unroll
      for (int kk = 0; kk < R / 32; kk++) {
        t.k[kk][blk] = load16_coherent(kplane + off + (uint32_t)(blk * (32 * R) + kk * 1024));
        t.v[kk][blk] = load16_coherent(vplane + off + (uint32_t)(blk * (32 * R) + kk * 1024));
      }
    const uint32_t moff = (uint32_t)tile * 64u + (uint32_t)lane;
    t.kmeta = __hip_atomic_load(kmeta + moff, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    t.vmeta = __hip_atomic_load(vmeta + moff, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}


// three limb dot products -> float: h*2^14 + m*2^7 + l
WSVD_DEV float limbs_to_f32(int h, int m, int l) { return fmaf((float)h, 16384.f, fmaf((float)m, 128.f, (float)l)); }

constexpr float kLimbFull = 1048576.f;    // 2^20: |quantised value| <= 2^20 fits three 7-bit limbs
constexpr int kMaxTilesPerFlush = 1024;   // 64 tokens * 127 * 127 per tile and limb: int32 holds > 2000 tiles

// NT = launch bound (threads); the workgroup may be launched with any multiple of 64 threads up to NT.
// STAGED: the variants that build something from B_K in LDS (rotary) or fold partial sums there (latent query) keep
// the staging areas; the plain kernel absorbs the query per wave on the matrix cores and needs none of them.
template <int R, int G, bool STAGED>
struct AttnStaging {
  v4i bk_lds[R * 128 * 2 / 16], bv_lds[R * 128 * 2 / 16];
  __attribute__((aligned(16))) float q_lds[G * 128];
  float qts[G * R];
};
template <int R, int G>
struct AttnStaging<R, G, false> {
  v4i bk_lds[1], bv_lds[1];
  float q_lds[1], qts[1];
};
template <int R, int G, int NT, bool STAGED = true>
struct AttnMfmaShared : AttnStaging<R, G, STAGED> {
  static constexpr int NWMAX = NT / 64;
  __attribute__((aligned(16))) int8_t qlimb[1][G][3][R];    // limbs of q~ in operand k-order
  float qdelta[G], qzsum[G];                                // unit of the limbs, sum of the quantised query
  __attribute__((aligned(16))) uint8_t wl[NWMAX][G][3][64]; // per wave: limbs of the value weights, by token
  __attribute__((aligned(16))) float wm[G][NWMAX], wls[G][NWMAX];   // per wave: running max (log2 domain), sum
  float wu[NWMAX][G * R + 1];                               // per wave: un-normalised latent-space accumulator [g][j];
                                                            // the odd row length keeps the merge's reads (lanes = waves) conflict-free
  float Msh[G], Lsh[G], Ush[G * R];
  int flag_sh;
};

// ---- rotary variant (reconstruct, rotate, then q K^T): extra state
// With a position rotation between K = C B_K and q K^T the factor cannot be folded into the query.  Regrouping
// the rotated product by frequency gives, for query position n-1 and key position t (i' = i + d/2):
//   s_t = sum_i cos(theta_i (n-1-t)) A_i(t) + sin(theta_i (n-1-t)) B_i(t),
//   A_i = q_i k_i + q_i' k_i',  B_i = q_i k_i' - q_i' k_i,   k = B_K^T c_t,
// and A_i, B_i are linear in the latent: [A; B](t) = N^T c_t with N (r x d) built once per (sequence, head) from
// q and B_K.  So the key tile is still "reconstructed" on the matrix cores, d outputs per token, straight from the
// cache stream (codes widened to fp16, exact; N carried as an fp16 pair hi + lo whose two products land in the same
// fp32 accumulator), and what is left per token is a dot product with its d position features, which each lane
// advances from block to block by a fixed rotation.
// N is scaled per frequency: the rows A_i and B_i share the unit delta_i = max |.| / 2^15 (so hi uses fp16's upper
// range and a lo that falls into the subnormals is below 2^-21 of the largest entry), and delta_i is folded into that
// frequency's features (delta_i cos, delta_i sin rotate like cos, sin), so it costs nothing per token.
// Row layout of the N^T operand: a 32-row MFMA block gives each half of the wave 16 rows = 16 features
// (row 8(v/4) + 4h + v%4 <-> accumulator register v); half h owns the frequencies [h d/4, (h+1) d/4), feature u of a
// half = frequency u/2, cosine (even u) or sine (odd u) term.  Contraction order of a 16-dim step: the lane of dim
// group g2 supplies dims 16 g2 + 8 s + e (step s of the pair, e < 8) - the bytes it already holds of the int8 image.
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
template <int D>
struct RopeGeom {
  static constexpr int NFH = D / 4;                 // frequencies per half wave
  static constexpr int NU = 2 * NFH;                // features per half wave
  static constexpr int NMB = NU / 16;               // 32-row operand blocks
};
template <int R, int G, int D>
struct RopeShared {
  // N^T as MFMA A operands: [head][operand block][16-dim step][hi, lo][lane][8]
  __attribute__((aligned(16))) _Float16 img[G][RopeGeom<D>::NMB][R / 16][2][512];
  float rot[2][D / 2][2];                           // cos, sin of theta_i * shift for the two block-to-block shifts
  uint32_t fmax_bits[D / 2];                        // per frequency: largest |entry| of its two rows over all heads
};
struct RopeArgs {
  uint32_t fq[64];                                  // theta_i / 2 pi as a 32-bit binary fraction of a revolution
  float rot[2][64][2];                              // cos, sin of theta_i * 32 and of theta_i * (64 * 8 - 32): the
                                                    // two block-to-block shifts of an 8-wave workgroup, from the host
};

// cos, sin of the angle `phase`, a 32-bit binary fraction of a revolution (the wrap-around of 32-bit arithmetic is
// the reduction mod 2 pi, exact), through the hardware's sine / cosine of an angle given in revolutions (a few 1e-7
// absolute error on [-1/2, 1/2)): used for the 2 x d/4 start values per lane
WSVD_DEV void phase_sincos_fast(uint32_t phase, float& c, float& s) {
  const float rev = (float)(int32_t)phase * (1.0f / 4294967296.0f);
  c = __builtin_amdgcn_cosf(rev);
  s = __builtin_amdgcn_sinf(rev);
}

// x * scale as an fp16 pair hi + lo.  The fp32 product is pinned in a register first: otherwise the compiler forms hi
// twice, once by rounding the fp32 product and once by rounding the exact product straight to fp16 (a fused
// multiply-convert), stores one and takes lo against the other; the two differ now and then by one fp16 step, which
// shows up as a 1e-4 error in single outputs.
WSVD_DEV void split_fp16_pair(float x, float scale, _Float16& hi, _Float16& lo) {
  float val = x * scale;
  asm volatile("" : "+v"(val));
  hi = (_Float16)val;
  lo = (_Float16)(val - (float)hi);
}

// One workgroup's share of the decode attention: kv head cx, context chunk cy, sequence cz.
// FUSED: the workgroup is part of a decode-step launch whose append workgroups are writing row seq_lens[b] at this
// very moment.  The row counts as present; the 64-row tile that contains it is kept out of the streaming loop and
// done last by one wave, after the two planes' flags show the launch's epoch, through agent-scope loads.
// ROPE_D != 0: the rotary variant for head dimension ROPE_D (rs, ra non-null).
// NEWROW: the second launch of the decode step.  The projection launch before it has advanced the lengths and left the
// new token's latents as partial sums; the workgroup whose chunk holds a sequence's last row sums them, quantises and
// stores the row (as the append would have) and patches it into the registers of the wave that consumes its tile.
template <int R, int G, bool I4, int NT, bool FUSED, int ROPE_D = 0, bool LATENT = false, bool PAGED = false, bool NEWROW = false>
WSVD_DEV void attn_mfma_body(const AttnParams& p, AttnMfmaShared<R, G, NT, (ROPE_D != 0 || LATENT)>& sh, const int cx, const int cy,
                             const int cz, RopeShared<R, G, (ROPE_D ? ROPE_D : 64)>* rs = nullptr, const RopeArgs* ra = nullptr) {
  constexpr bool ROPE = ROPE_D != 0;
  constexpr bool STAGED = ROPE || LATENT;
  using RG = RopeGeom<(ROPE_D ? ROPE_D : 64)>;
  static_assert(!ROPE || !FUSED, "rotary variant: stand-alone launch");
  static_assert(!LATENT || (!ROPE && !FUSED), "latent-query variant: stand-alone launch, no rotation");
  static_assert(!I4 || R == 32, "int4 latents: rank 32 only");
  static_assert(!PAGED || (!ROPE && !LATENT && !FUSED), "paged cache: the plain decode attention");
  static_assert(!NEWROW || (!ROPE && !LATENT && !FUSED && !PAGED && !I4), "deferred row: the plain int8 decode attention");
  static_assert(G >= 1 && G <= 4, "paired-block kernel handles up to 4 query heads per kv head");
  constexpr int KK = R / 32;
  constexpr int NWMAX = NT / 64;
  constexpr int FIT = R / 16;           // 16-byte staging passes for an R x 128 bf16 factor
  auto& bk_lds = sh.bk_lds; auto& bv_lds = sh.bv_lds; auto& q_lds = sh.q_lds; auto& qts = sh.qts; auto& qlimb = sh.qlimb;
  auto& qdelta = sh.qdelta; auto& qzsum = sh.qzsum; auto& wl = sh.wl; auto& wm = sh.wm; auto& wls = sh.wls; auto& wu = sh.wu;
  auto& Msh = sh.Msh; auto& Lsh = sh.Lsh; auto& Ush = sh.Ush; int& flag_sh = sh.flag_sh;

  // scalar loads first: issued ahead of the flood of vector loads they come back quickly, and nothing needs them
  // until the tile loop
  const int n_raw = p.seq_lens[cz];
  [[maybe_unused]] const int pend_raw = NEWROW ? p.pending[cz] : 0;
  const uint32_t qs_raw = q_scale_raw(p, cz);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NW = blockDim.x >> 6;
  // NEWROW: the row stored by this launch (K | V codes and scales): written by wave 1 or 2, read by the
  // wave that consumes the row's tile once new_ready says so
  __shared__ __attribute__((aligned(16))) uint8_t new_codes[2][NEWROW ? R : 16];
  __shared__ uint16_t new_scale[2];
  __shared__ int new_ready;
  if (NEWROW && tid == 0) new_ready = 0;          // (ordered before its first use by the workgroup barrier below)
  __builtin_amdgcn_s_setprio(3);          // streaming waves first (see the end of the tile loop)
  [[maybe_unused]] long long* const tl = FUSED ? nullptr : p.timeline;
  [[maybe_unused]] const int tl_wg = (cz * (int)gridDim.y + cy) * (int)gridDim.x + cx;
  WSVD_STAMP(tl, tl_wg, wave, 0);
  const size_t ph = (size_t)cz * p.Hkv + cx;
  const size_t plane_bytes = (size_t)p.t_cap * (I4 ? R / 2 : R);
  const uint8_t* kplane = p.k_codes + ph * plane_bytes;
  const uint8_t* vplane = p.v_codes + ph * plane_bytes;
  const uint16_t* kmeta = p.k_meta + ph * (size_t)p.t_cap * (I4 ? 2 : 1);
  const uint16_t* vmeta = p.v_meta + ph * (size_t)p.t_cap * (I4 ? 2 : 1);
  // Paged cache: rows [i * page_rows, (i + 1) * page_rows) of sequence b live in page block_table[b][i] of the pools,
  // a page holding that row range of every kv head in the layout of the contiguous planes.  A tile (64 rows) never
  // straddles pages.  Entries that are out of range (pages past the sequence's end may hold anything, and tiles are
  // requested before the length is known) are read as page 0: such tiles are never consumed.
  // The table entries of this workgroup's chunk are fetched once, one per lane, with the first loads of the kernel; a
  // tile's entry is then a lane read (the tile index is wave-uniform), not a dependent trip to memory per tile.
  [[maybe_unused]] int page_entry = 0, page0 = 0;
  if constexpr (PAGED) {
    const int tpp = p.page_rows >> 6;
    page0 = ((int)cy * (p.chunk_rows >> 6)) / tpp;
    page_entry = p.block_table[(size_t)cz * p.max_pages + min(page0 + lane, p.max_pages - 1)];
  }
  auto tile_load = [&](TileRegs<R, I4>& t, int tile, int which /* 0 both, 1 K side, 2 V side */) {
    const uint8_t *kp = kplane, *vp = vplane;
    const uint16_t *km = kmeta, *vm = vmeta;
    int ti = tile;
    if constexpr (PAGED) {
      const int tpp = p.page_rows >> 6;
      const int pg = min(tile / tpp, p.max_pages - 1);
      const int rel = __builtin_amdgcn_readfirstlane(pg - page0);
      int phys = (rel >= 0 && rel < 64) ? __builtin_amdgcn_readlane(page_entry, rel)
                                        : p.block_table[(size_t)cz * p.max_pages + pg];     // (chunks of more than 64 pages)
      phys = (phys >= 0 && phys < p.n_pages) ? phys : 0;
      const size_t slot = (size_t)phys * p.Hkv + cx;
      const size_t pb = (size_t)p.page_rows * (I4 ? R / 2 : R), pm = (size_t)p.page_rows * (I4 ? 2 : 1);
      kp = p.k_codes + slot * pb; vp = p.v_codes + slot * pb;
      km = p.k_meta + slot * pm; vm = p.v_meta + slot * pm;
      ti = tile - pg * tpp;
    }
    if (which != 2) load_tile_k<R, I4>(t, kp, km, ti, lane);
    if (which != 1) load_tile_v<R, I4>(t, vp, vm, ti, lane);
  };

  // ---- loads, in the order they should come back: the small per-head inputs first, then DEPTH tiles per wave (a
  // tile = 64 rows of K and V codes plus metadata), requested before the sequence length is known.  Every tile below
  // t_cap is allocated memory, so the loads are safe; tiles past the sequence end are never consumed.  The prologue
  // below then runs in the shadow of the first tiles' latency.
  constexpr int DEPTH = 2;   // deeper prefetch costs registers and measured slower
  TileRegs<R, I4> buf[DEPTH];
  const int chunk_tiles = p.chunk_rows >> 6;
  int T = (int)cy * chunk_tiles + wave;
  // unconditional (clamped to the chunk's last allocated tile): see stage_issue
  const int spec_last = min(((int)cy + 1) * chunk_tiles, p.t_cap >> 6) - 1;
  constexpr int MAXP = 4;                                        // NEWROW: partial sums per latent element, at most
  // rank 32: lanes 0..31 carry the K row's dims, lanes 32..63 the V row's (np_a); rank 64: np_a = K, np_b = V
  [[maybe_unused]] float np_a[NEWROW ? MAXP : 1], np_b[NEWROW && R == 64 ? MAXP : 1];
  [[maybe_unused]] bool nr_mine = false;
  if constexpr (!STAGED) {
    // Query absorption q~ = c_scale * B_K q on the matrix cores, by the workgroup's first wave alone, operands
    // straight from memory (no staging in LDS): 8-16 KB of B_K and the queries are the only small loads of the
    // workgroup, they sit at the head of that wave's queue, and a single barrier hands the limbs to the other waves,
    // whose first tiles are in flight by then.  (Every wave absorbing for itself needs no barrier at all, but puts
    // the whole factor through the CU's address pipeline once per wave, ahead of the tiles: measured slower.)
    // D[i][j] = sum_k A[i][k] B[k][j] with V_MFMA_F32_32X32X16_BF16: column j = latent dim (B = B_K^T, a lane's 8
    // operand elements are 16 contiguous bytes of row j of B_K), row i = 8 g + part: the contraction over the head
    // dim is cut into d/16 parts of 16 (8 per half wave), row (g, part) carries q_g only in MFMA step `part` and
    // zeros otherwise, so each lane needs just the 8 query elements of its own (g, part, half) and the parts add up
    // afterwards: 4 accumulator registers plus one exchange between the half waves.
    // Contraction order: step ks, half h, element e <-> head dim (d/2) h + 8 ks + e.
    const int l32 = lane & 31, hf = lane >> 5;
    const int nks = p.d >> 4;                                     // 8 (d = 128) or 4
    const int qg = l32 >> 3, qpart = l32 & 7;                     // this lane's row: query slot, part
    const bool qrow_on = qg < G && qpart < nks;
    const bool leader = wave == 0;                                // wave-uniform
    v4i bkr[KK][8];
    v4i q_raw[2];
    // the lane's 8 query elements: 8, 16 or 32 bytes inside one or two aligned 16-byte pieces
    const int q_esz = p.q_dtype == WSVD_F32 ? 4 : p.q_dtype == WSVD_BF16 ? 2 : 1;
    const size_t q_elem = ((size_t)cz * p.Hq + first_head(p, cx) + (qrow_on ? qg : 0)) * p.d + (p.d >> 1) * hf + 8 * (qrow_on ? qpart : 0);
    const size_t q_off = q_elem * q_esz, q_o0 = q_off & ~(size_t)15;
    const size_t q_bytes = (size_t)p.B * p.Hq * p.d * q_esz;
    if (leader) {
#pragma unroll
    for (int jb = 0; jb < KK; jb++)
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        const int c = (p.d >> 1) * hf + 8 * min(ks, nks - 1);     // clamped
        bkr[jb][ks] = *(const v4i*)((const char*)p.BK + (((size_t)cx * R + 32 * jb + l32) * p.d + c) * 2);
      }
    q_raw[0] = *(const v4i*)((const char*)p.q + q_o0);
    q_raw[1] = *(const v4i*)((const char*)p.q + min(q_o0 + 16, q_bytes - 16));
    }
    // NEWROW: waves 1 and 2 ask for the partial sums of their (sequence, kv head) now, ahead of the tiles and
    // whether or not the row turns out to be this workgroup's (the addresses do not depend on the length).  They were
    // written by the launch before this one, on other XCDs: they come from memory, not from this XCD's L2
    if constexpr (NEWROW) {
      if (wave == 1 || wave == 2) {
        const float* src = (R == 32 && lane >= 32) ? p.new_v : p.new_k;
        const size_t o = (size_t)cz * p.new_ld + (size_t)cx * R + (lane & (R - 1));
        // straight-line, clamped (a surplus slot repeats the last part and is left out of the sum): loads under
        // branches made the compiler wait for them on the spot, in front of the barrier below
#pragma unroll
        for (int sidx = 0; sidx < MAXP; sidx++) {
          const size_t po = (size_t)min(sidx, p.n_parts - 1) * p.part_stride + o;
          np_a[sidx] = src[po];
          if constexpr (R == 64) np_b[sidx] = p.new_v[po];
        }
      }
    }
    // The barrier (no memory wait) puts the leader's small loads ahead of every wave's tile loads in the CU's address
    // pipeline: the first two tiles of 16 waves are 190 KB of requests, more than a microsecond of that pipeline, and
    // the absorption must not queue behind them.
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < DEPTH; i++) tile_load(buf[i], min(T + i * NW, spec_last), 0);
    WSVD_STAMP(tl, tl_wg, wave, 1);

    if (leader) {
    float f[8];
    if (p.q_dtype == WSVD_F32) {
#pragma unroll
      for (int e = 0; e < 4; e++) { f[e] = __int_as_float(q_raw[0][e]); f[4 + e] = __int_as_float(q_raw[1][e]); }
    } else if (p.q_dtype == WSVD_BF16) {
#pragma unroll
      for (int e = 0; e < 4; e++) {
        f[2 * e] = __uint_as_float((uint32_t)q_raw[0][e] << 16);
        f[2 * e + 1] = __uint_as_float((uint32_t)q_raw[0][e] & 0xFFFF0000u);
      }
    } else {                                                      // int8: 8 bytes, the low or the high half of the piece
      const bool hi = (q_off & 8) != 0;
      const uint32_t d0 = (uint32_t)(hi ? q_raw[0][2] : q_raw[0][0]), d1 = (uint32_t)(hi ? q_raw[0][3] : q_raw[0][1]);
#pragma unroll
      for (int e = 0; e < 4; e++) { f[e] = (float)(int8_t)(d0 >> (8 * e)); f[4 + e] = (float)(int8_t)(d1 >> (8 * e)); }
    }
    if (!qrow_on) {
#pragma unroll
      for (int e = 0; e < 8; e++) f[e] = 0.f;
    }
    // bf16 terms of the query chunk: one is exact for bf16 and int8 queries, an fp32 query takes three (hi + mid + lo
    // reproduces it to 2^-24)
    const int n_terms = p.q_dtype == WSVD_F32 ? 3 : 1;
    v16f qacc[KK];
#pragma unroll
    for (int jb = 0; jb < KK; jb++)
#pragma unroll
      for (int x = 0; x < 16; x++) qacc[jb][x] = 0.f;
    for (int t3 = 0; t3 < n_terms; t3++) {
      v4i packed;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const uint32_t h0 = __float_as_uint(f[2 * e]) & 0xFFFF0000u, h1 = __float_as_uint(f[2 * e + 1]) & 0xFFFF0000u;
        packed[e] = (int)((h0 >> 16) | h1);
        f[2 * e] -= __uint_as_float(h0);                          // exact: the remainder has at most 16 significant bits
        f[2 * e + 1] -= __uint_as_float(h1);
      }
      const v4i zero4 = {0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        if (ks < nks) {                                           // wave-uniform
          const v8bf a_op = __builtin_bit_cast(v8bf, qpart == ks ? packed : zero4);
#pragma unroll
          for (int jb = 0; jb < KK; jb++)
            qacc[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_op, __builtin_bit_cast(v8bf, bkr[jb][ks]), qacc[jb], 0, 0, 0);
        }
      }
    }
    // D row 8 g + part sits in register 4 g + part % 4 of half part / 4: add the four registers, then the two halves
    // (after which lane L and lane L ^ 32 both hold q~[g][32 jb + L % 32])
    float qt[G][KK];
#pragma unroll
    for (int g = 0; g < G; g++)
#pragma unroll
      for (int jb = 0; jb < KK; jb++) {
        const float part = (qacc[jb][4 * g] + qacc[jb][4 * g + 1]) + (qacc[jb][4 * g + 2] + qacc[jb][4 * g + 3]);
        qt[g][jb] = (part + __shfl_xor(part, 32)) * p.c_scale;
      }
#pragma unroll
    for (int g = 0; g < G; g++) {
      float am = 0.f;
#pragma unroll
      for (int jb = 0; jb < KK; jb++) am = fmaxf(am, fabsf(qt[g][jb]));
      const float amax = half_max(am, lane);                      // both halves hold all dims
      const float inv = amax > 0.f ? kLimbFull / amax : 0.f;
      float qsum = 0.f;
#pragma unroll
      for (int jb = 0; jb < KK; jb++) {
        const int Q = (int)__builtin_rintf(qt[g][jb] * inv);
        const int l0 = ((Q + 64) & 127) - 64;                     // balanced digits, each in [-64, 64]
        const int Q1 = (Q - l0) >> 7;
        const int l1 = ((Q1 + 64) & 127) - 64;
        const int l2 = (Q1 - l1) >> 7;
        qsum += (float)Q;
        // position of dim j in the operand k-order.  I8: identity.  I4: a lane's 8 bytes hold dims 16g..16g+15 as
        // nibble pairs; masking gives operand dwords [even dims 0..6, odd 1..7, even 8..14, odd 9..15].
        const int j = 32 * jb + l32;
        int pos = j;
        if (I4) {
          const int jj = j & 15;
          pos = (j & 16) + ((jj >> 3) << 3) + ((jj & 1) << 2) + ((jj & 7) >> 1);
        }
        if (hf == 0) {
          qlimb[0][g][0][pos] = (int8_t)l2;
          qlimb[0][g][1][pos] = (int8_t)l1;
          qlimb[0][g][2][pos] = (int8_t)l0;
        }
      }
      const float zs = I4 ? half_sum(qsum, lane) : 0.f;
      if (lane == 0) { qdelta[g] = amax > 0.f ? amax / kLimbFull : 0.f; qzsum[g] = zs; }
    }
    }   // leader
    __syncthreads();
    WSVD_STAMP(tl, tl_wg, wave, 3);
    if constexpr (NEWROW) {
      // The row, by one wave, off everybody else's path: the other waves go on to their tiles, the wave that
      // consumes the row's tile (its last one) looks at new_ready when it gets there.
      // (A sequence longer than the caller's bound is reported by decode_work; its row is still stored, by the last chunk.)
      // The producer is wave 1, or wave 2 when wave 1 is the tile's consumer: both have asked for the partial sums; the
      // early waves of a workgroup get their tiles first and finish first, so the row's work costs the workgroup nothing
      // there (on the last wave it made that wave the workgroup's last by 0.8 us).
      if (wave == 1 || wave == 2) {
        const int row = n_raw - 1, ct = p.chunk_rows >> 6, cyo = min((row >> 6) / ct, p.n_chunks - 1);
        const int consumer = ((row >> 6) - cyo * ct) % NW;
        if (pend_raw != 0 && n_raw >= 1 && n_raw <= p.t_cap && (int)cy == cyo && wave == (consumer == 1 ? 2 : 1)) {       // wave-uniform
          // (the empty statements pin the first use of the loaded values here: hoisted to the loads, the first
          // addition made the whole workgroup wait for them in front of the barrier above)
#pragma unroll
          for (int sidx = 0; sidx < MAXP; sidx++) {
            asm volatile("" : "+v"(np_a[sidx]));
            if constexpr (R == 64) asm volatile("" : "+v"(np_b[sidx]));
          }
          // The cache row for later launches (the rule and the layout of the append kernels' row store), and a copy in
          // LDS for this one: the tile that holds the row is fetched like any other, possibly before these stores land;
          // its consumer overwrites the row's bytes in registers.  One pass with both rows side by side at rank 32.
          const int j = lane & (R - 1);
#pragma unroll
          for (int pass = 0; pass < (R == 32 ? 1 : 2); pass++) {
            const int pl = R == 32 ? (lane >> 5) : pass;
            float c = 0.f;
#pragma unroll
            for (int sidx = 0; sidx < MAXP; sidx++)                    // slice order
              c += sidx < p.n_parts ? (pass == 0 ? np_a[sidx] : np_b[R == 64 ? sidx : 0]) : 0.f;
            const float a = R == 64 ? wave_max(fabsf(c)) : half_max(fabsf(c), lane);
            uint16_t sh16 = 0x3C00u;
            if (a != 0.f) sh16 = guard_scale_f16(a / 127.0f);
            const float sc = f16_bits_to_f32(sh16);
            const uint8_t code = (uint8_t)(int8_t)(int)fminf(fmaxf(__builtin_rintf(c / sc), -127.f), 127.f);
            uint8_t* plane = const_cast<uint8_t*>(pl ? p.v_codes : p.k_codes) + ph * plane_bytes;
            plane[pl ? i8_v_offset(row, j, R) : i8_k_offset(row, j, R)] = code;
            if (j == 0) const_cast<uint16_t*>(pl ? p.v_meta : p.k_meta)[ph * (size_t)p.t_cap + row] = sh16;
            new_codes[pl][j] = code;
            if (j == 0) new_scale[pl] = sh16;
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
          if (lane == 0) __hip_atomic_store(&new_ready, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      }
    }
  } else {
  const int fac16 = R * p.d * 2 / 16;
  StageRegs<FIT> stk, stv;
  QRegs qr;
  // LATENT: q~[g][j] = sum_i c_Q[g][i] (B_Q B_K^T)[h][i][j].  Work item (quarter of the i range, g, j), j fastest so
  // that a wave's loads of the fold are contiguous; up to 16 products per item, the quarters meet in LDS.
  constexpr int LQ = 16;                               // rq <= 64
  constexpr int NLP = LATENT ? (4 * G * R + 255) / 256 : 1;   // passes at the smallest workgroup (256 threads)
  float lat_part[NLP];
  if constexpr (LATENT) {
    const int qn = (p.rq + 3) >> 2;                    // i values per quarter
#pragma unroll
    for (int ps = 0; ps < NLP; ps++) {
      const int item = min(tid + ps * (int)blockDim.x, 4 * G * R - 1);
      const int j = item % R, g = (item / R) % G, part = item / (R * G);
      const int h = (int)first_head(p, cx) + g;
      const float* cq = (const float*)p.q + ((size_t)cz * p.Hq + h) * p.rq;
      const float* fold = p.qk_fold + (size_t)h * p.rq * R + j;
      float mv[LQ], cv[LQ];
#pragma unroll
      for (int ii = 0; ii < LQ; ii++) {
        const int i = min(part * qn + ii, p.rq - 1);   // clamped: surplus slots are masked below
        mv[ii] = fold[(size_t)i * R];
        cv[ii] = cq[i];
      }
      float acc = 0.f;
#pragma unroll
      for (int ii = 0; ii < LQ; ii++) acc = (ii < qn && part * qn + ii < p.rq) ? fmaf(cv[ii], mv[ii], acc) : acc;
      lat_part[ps] = acc;
    }
  } else {
  stage_issue<FIT>(stk, (const char*)p.BK + (size_t)cx * R * p.d * 2, fac16);
  stage_issue<FIT>(stv, (const char*)p.BV + (size_t)cx * R * p.d * 2, fac16);
  q_issue(p, cz, cx, qr);
  }
#pragma unroll
  for (int i = 0; i < DEPTH; i++) load_tile<R, I4>(buf[i], kplane, vplane, kmeta, vmeta, min(T + i * NW, spec_last), lane);
  WSVD_STAMP(tl, tl_wg, wave, 1);

  // ---- query absorption and its limbs
  if constexpr (LATENT) {
    float* qpart = (float*)bk_lds;       // [4][G*R] partial sums (B_K is not staged in this variant)
#pragma unroll
    for (int ps = 0; ps < NLP; ps++) {
      const int item = tid + ps * (int)blockDim.x;
      if (item < 4 * G * R) qpart[item] = lat_part[ps];
    }
    __syncthreads();
    if (tid < G * R) qts[tid] = (qpart[tid] + qpart[G * R + tid] + qpart[2 * G * R + tid] + qpart[3 * G * R + tid]) * p.c_scale;
  } else {
  stage_commit<FIT>(stk, bk_lds, fac16);
  stage_commit<FIT>(stv, bv_lds, fac16);
  q_commit(p, qr, 1.f, q_lds);          // an int8 query's scale is applied to delta below
  }
  __syncthreads();
  WSVD_STAMP(tl, tl_wg, wave, 2);
  if constexpr (ROPE) {
    constexpr int Dh = ROPE_D / 2;
    // block-to-block rotations: +32 tokens (second block of a tile), then on to the wave's next tile
    if (tid < 2 * Dh) {
      const int which = tid / Dh, i = tid % Dh;
      rs->rot[which][i][0] = ra->rot[which][i][0]; rs->rot[which][i][1] = ra->rot[which][i][1];
    }
    // N (r x d per query head), written as whole 16-byte operand slots: a slot = one feature row (head, cosine or
    // sine term, frequency i) x 8 consecutive latent dims.  Consecutive threads take consecutive frequencies.
    const uint16_t* bk16 = (const uint16_t*)bk_lds;
    constexpr int NSLOT = G * 2 * (R / 8) * Dh;
    constexpr int NS = (NSLOT + NT - 1) / NT;           // slots per thread; the launch uses exactly NT threads
    for (int i = tid; i < Dh; i += NT) rs->fmax_bits[i] = 0u;
    float ent[NS][8];
#pragma unroll
    for (int k = 0; k < NS; k++) {
      const int slot = min(tid + k * NT, NSLOT - 1);    // surplus threads repeat the last slot and do not write
      const int fi = slot % Dh, jgrp = (slot / Dh) % (R / 8), type = (slot / (Dh * (R / 8))) % 2, g = slot / (Dh * (R / 8) * 2);
      const float qi = q_lds[g * ROPE_D + fi] * p.c_scale, qj = q_lds[g * ROPE_D + fi + Dh] * p.c_scale;
      // cosine term: q_i k_i + q_i' k_i';  sine term: q_i k_i' - q_i' k_i
      const float wa = type ? -qj : qi, wb = type ? qi : qj;
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const int j = 8 * jgrp + e;
        ent[k][e] = fmaf(wa, bf16_to_f32(bk16[j * ROPE_D + fi]), wb * bf16_to_f32(bk16[j * ROPE_D + fi + Dh]));
      }
    }
    __syncthreads();                                     // fmax_bits cleared
#pragma unroll
    for (int k = 0; k < NS; k++) {
      float mx = 0.f;
#pragma unroll
      for (int e = 0; e < 8; e++) mx = fmaxf(mx, fabsf(ent[k][e]));
      const int slot = min(tid + k * NT, NSLOT - 1);
      atomicMax(&rs->fmax_bits[slot % Dh], __float_as_uint(mx));   // non-negative floats order like their bits
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NS; k++) {
      const int slot = tid + k * NT;
      if (slot < NSLOT) {
        const int fi = slot % Dh, jgrp = (slot / Dh) % (R / 8), type = (slot / (Dh * (R / 8))) % 2, g = slot / (Dh * (R / 8) * 2);
        const float amax = __uint_as_float(rs->fmax_bits[fi]);
        const float inv = amax > 0.f ? 32768.f / amax : 0.f;
        const int hh = fi / RG::NFH, uu = 2 * (fi % RG::NFH) + type;         // half, feature within the half
        const int mb = uu >> 4, v = uu & 15;
        const int row = 8 * (v >> 2) + 4 * hh + (v & 3);
        const int ks = ((jgrp >> 2) << 1) | (jgrp & 1), g2 = (jgrp >> 1) & 1;
        v8h hi, lo;
#pragma unroll
        for (int e = 0; e < 8; e++) {
          _Float16 h, l;
          split_fp16_pair(ent[k][e], inv, h, l);
          hi[e] = h; lo[e] = l;
        }
        *(v8h*)&rs->img[g][mb][ks][0][(g2 * 32 + row) * 8] = hi;
        *(v8h*)&rs->img[g][mb][ks][1][(g2 * 32 + row) * 8] = lo;
      }
    }
    if (tid < G) qdelta[tid] = 1.f;
  } else {
  if constexpr (!LATENT) compute_qtilde<R, 2>(p, bk_lds, q_lds, qts);
  if (tid < G * R) {
    const int g = tid / R, j = tid % R;
    const float v = qts[tid];
    const float amax = (R == 64) ? wave_max(fabsf(v)) : half_max(fabsf(v), lane);
    const float inv = amax > 0.f ? kLimbFull / amax : 0.f;
    const int Q = (int)__builtin_rintf(v * inv);
    const int l0 = ((Q + 64) & 127) - 64;          // balanced digits, each in [-64, 64]
    const int Q1 = (Q - l0) >> 7;
    const int l1 = ((Q1 + 64) & 127) - 64;
    const int l2 = (Q1 - l1) >> 7;
    // position of dim j in the operand k-order.  I8: identity.  I4: a lane's 8 bytes hold dims 16g..16g+15 as
    // nibble pairs; masking gives operand dwords [even dims 0..6, odd 1..7, even 8..14, odd 9..15].
    int pos = j;
    if (I4) {
      const int jj = j & 15;
      pos = (j & 16) + ((jj >> 3) << 3) + ((jj & 1) << 2) + ((jj & 7) >> 1);
    }
    qlimb[0][g][0][pos] = (int8_t)l2;
    qlimb[0][g][1][pos] = (int8_t)l1;
    qlimb[0][g][2][pos] = (int8_t)l0;
    const float zs = (R == 64) ? wave_sum((float)Q) : half_sum((float)Q, lane);
    if (j == 0) { qdelta[g] = amax > 0.f ? amax / kLimbFull : 0.f; qzsum[g] = zs; }
  }
  }
  __syncthreads();
  WSVD_STAMP(tl, tl_wg, wave, 3);

  }   // STAGED

  // A operands of the score MFMAs.  Row i of A: query slot a = i/8, row group (i/4)%2, limb i%4 (limb 3 unused).
  // a1 feeds block 0 of a tile (rows of group 0 only), a2 feeds block 1 (rows of group 1 only).
  v4i a1[KK], a2[KK];
  if constexpr (!ROPE) {
    const int i = lane & 31, g2 = lane >> 5;
    const int a = i >> 3, grp = (i >> 2) & 1, limb = i & 3;
    const bool act = (a < G) && (limb < 3);
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      const v4i val = *(const v4i*)&qlimb[0][a < G ? a : 0][limb < 3 ? limb : 0][kk * 32 + g2 * 16];
      const v4i zero = {0, 0, 0, 0};
      a1[kk] = (act && grp == 0) ? val : zero;
      a2[kk] = (act && grp == 1) ? val : zero;
    }
  }

  // only now are the sequence length and the query scale needed
  const float qs = q_scale_value(p, cz, qs_raw);
  const bool has_new = FUSED && n_raw >= 0 && n_raw < p.t_cap;          // the row being appended by this launch
  const WorkItem w = decode_work(p, n_raw + (has_new ? 1 : 0), cx, cy, cz);
  if (w.n == 0) { write_zero_outputs(p, w); return; }
  if (!w.active) return;
  const int new_tile = n_raw >> 6;                                      // tile of the new row (its chunk's last tile)
  const bool own_new = has_new && new_tile >= cy * chunk_tiles && new_tile < (cy + 1) * chunk_tiles;
  const int tile_end = ((w.row_end + 63) >> 6) - (own_new ? 1 : 0);
  [[maybe_unused]] const int nr_row = n_raw - 1, nr_tile = nr_row >> 6;
  if constexpr (NEWROW)
    nr_mine = pend_raw != 0 && n_raw >= 1 && n_raw <= p.t_cap && nr_tile >= cy * chunk_tiles && nr_tile < (cy + 1) * chunk_tiles;
  float delta[G], zsum[G];
#pragma unroll
  for (int g = 0; g < G; g++) {
    delta[g] = qdelta[g] * qs;
    zsum[g] = I4 ? qzsum[g] : 0.f;
  }

  // rotary variant: this lane's position features (its token of the current block, the frequencies of its half)
  float fc[ROPE ? RG::NFH : 1], fs[ROPE ? RG::NFH : 1];
  if constexpr (ROPE) {
    const int hf = lane >> 5;
    const uint32_t dist = (uint32_t)(n_raw - 1 - (T * 64 + (lane & 31)));   // query position minus key position
#pragma unroll
    for (int i = 0; i < RG::NFH; i++) {
      phase_sincos_fast(ra->fq[hf * RG::NFH + i] * dist, fc[i], fs[i]);
      const float unit = __uint_as_float(rs->fmax_bits[hf * RG::NFH + i]) * (1.0f / 32768.f);
      fc[i] *= unit; fs[i] *= unit;
    }
  }
  // advance the features by one of the two block-to-block shifts: the distance shrinks, so the angle turns back
  auto rope_advance = [&](int which) {
    if constexpr (ROPE) {
      const int hf = lane >> 5;
#pragma unroll
      for (int i = 0; i < RG::NFH; i += 2) {
        const v4f r4 = *(const v4f*)&rs->rot[which][hf * RG::NFH + i][0];    // (cos, sin) of two frequencies
        const float c0 = fc[i], s0 = fs[i], c1 = fc[i + 1], s1 = fs[i + 1];
        fc[i] = fmaf(c0, r4[0], s0 * r4[1]);      fs[i] = fmaf(s0, r4[0], -(c0 * r4[1]));
        fc[i + 1] = fmaf(c1, r4[2], s1 * r4[3]);  fs[i + 1] = fmaf(s1, r4[2], -(c1 * r4[3]));
      }
    }
  };

  // running state: m (log2-domain reference), wref (fixed-point range of the value weights), their derived
  // omega = wref / 2^20 and winv = 2^20 / wref; lsum, zacc, u are per-lane partial sums
  float m[G], wref[G], omega[G], winv[G], lsum[G], zacc[G], u[G][KK];
  v16i vacc[KK];
#pragma unroll
  for (int g = 0; g < G; g++) {
    m[g] = -INFINITY; wref[g] = 0.f; omega[g] = 0.f; winv[g] = 0.f; lsum[g] = 0.f; zacc[g] = 0.f;
#pragma unroll
    for (int jj = 0; jj < KK; jj++) u[g][jj] = 0.f;
  }
#pragma unroll
  for (int jj = 0; jj < KK; jj++)
#pragma unroll
    for (int x = 0; x < 16; x++) vacc[jj][x] = 0;
  int since_flush = 0;

  // int32 accumulators of head slot g -> float accumulators, in units of the current omega
  auto flush = [&](int g) {
#pragma unroll
    for (int jj = 0; jj < KK; jj++) {
      u[g][jj] = fmaf(omega[g], limbs_to_f32(vacc[jj][4 * g], vacc[jj][4 * g + 1], vacc[jj][4 * g + 2]), u[g][jj]);
      vacc[jj][4 * g] = 0; vacc[jj][4 * g + 1] = 0; vacc[jj][4 * g + 2] = 0;
    }
  };

  // weights operand read position: row i -> (query slot, limb); both row groups read the same limbs
  const int wr_a = min((lane & 31) >> 3, G - 1), wr_limb = min(lane & 3, 2), wr_g2 = lane >> 5;
  // token order inside the wave's limb rows.  I8: token L at byte L.  I4: a V byte holds tokens (2b, 2b+1) of a
  // 32-token half; the low-nibble operand covers even tokens, the high-nibble operand odd tokens.
  const int wpos = I4 ? ((lane & 1) << 5) + ((lane >> 5) << 4) + ((lane & 31) >> 1) : lane;

#ifdef WSVD_TIMELINE
  bool tl_first = true;
#endif
  // refill: std::true_type = request tile `next` into the same registers as they fall free, the key side right after
  // the score products, the value side at the end
  auto compute = [&](auto refill, TileRegs<R, I4>& t, int tile, int next) {
    const bool valid = tile * 64 + lane < w.row_end;
    if constexpr (NEWROW) {
      if (nr_mine && tile == nr_tile) {                    // wave-uniform: put the row stored by this launch into the tile
        int budget = 1 << 20;                              // (the last wave wrote it microseconds ago; the bound keeps the kernel finite)
        while (__hip_atomic_load(&new_ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0 && budget > 0) {
          __builtin_amdgcn_s_sleep(2);
          budget--;
        }
        if (budget == 0 && lane == 0) atomicExch(p.err_word, (int)WSVD_E_HIP);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int ti = nr_row & 63, blk = ti >> 5, tn = ti & 31;
        const int l32 = lane & 31, hf = lane >> 5;
#pragma unroll
        for (int b2 = 0; b2 < 2; b2++) {
          if (b2 == blk) {
#pragma unroll
            for (int kk = 0; kk < KK; kk++) {
              // K: lane (token tn, dim half hf) holds dims 32 kk + 16 hf .. + 15 of its token
              if (l32 == tn) t.k[kk][b2] = *(const v4i*)&new_codes[0][32 * kk + 16 * hf];
              // V: lane (dim 32 kk + l32, token half hf) holds 16 tokens of its dim: byte tn % 16 of the half tn / 16
              if (hf == (tn >> 4)) {
                const uint32_t byte = new_codes[1][32 * kk + l32];
                const int dw = (tn & 15) >> 2, sh8 = 8 * (tn & 3);
#pragma unroll
                for (int e = 0; e < 4; e++)
                  if (e == dw) t.v[kk][b2][e] = (int)(((uint32_t)t.v[kk][b2][e] & ~(0xFFu << sh8)) | (byte << sh8));
              }
            }
          }
        }
        if (lane == ti) { t.kmeta = new_scale[0]; t.vmeta = new_scale[1]; }
      }
    }
    // ---------------- score pass
    v16i acc = {0};
    float ksc, kz = 0.f, vsc, vz = 0.f;
    if constexpr (ROPE && I4) {
      ksc = f16_bits_to_f32((uint16_t)(t.kmeta & 0xFFFF)); kz = f16_bits_to_f32((uint16_t)(t.kmeta >> 16));
      vsc = f16_bits_to_f32((uint16_t)(t.vmeta & 0xFFFF)); vz = f16_bits_to_f32((uint16_t)(t.vmeta >> 16));
    } else if (I4) {
      const uint32_t msk = 0x0F0F0F0Fu;
      const v4i raw = t.k[0][0];
      v4i s0, s1;   // slot 0 = tokens 0..31 (dwords 0,1), slot 1 = tokens 32..63 (dwords 2,3)
      s0[0] = raw[0] & msk; s0[1] = ((uint32_t)raw[0] >> 4) & msk; s0[2] = raw[1] & msk; s0[3] = ((uint32_t)raw[1] >> 4) & msk;
      s1[0] = raw[2] & msk; s1[1] = ((uint32_t)raw[2] >> 4) & msk; s1[2] = raw[3] & msk; s1[3] = ((uint32_t)raw[3] >> 4) & msk;
      acc = mfma_i8(a1[0], s0, acc);
      acc = mfma_i8(a2[0], s1, acc);
      ksc = f16_bits_to_f32((uint16_t)(t.kmeta & 0xFFFF)); kz = f16_bits_to_f32((uint16_t)(t.kmeta >> 16));
      vsc = f16_bits_to_f32((uint16_t)(t.vmeta & 0xFFFF)); vz = f16_bits_to_f32((uint16_t)(t.vmeta >> 16));
    } else if constexpr (ROPE) {
      ksc = f16_bits_to_f32((uint16_t)t.kmeta);
      vsc = f16_bits_to_f32((uint16_t)t.vmeta);
    } else {
#pragma unroll
      for (int kk = 0; kk < KK; kk++) acc = mfma_i8(a1[kk], t.k[kk][0], acc);
#pragma unroll
      for (int kk = 0; kk < KK; kk++) acc = mfma_i8(a2[kk], t.k[kk][1], acc);
      ksc = f16_bits_to_f32((uint16_t)t.kmeta);
      vsc = f16_bits_to_f32((uint16_t)t.vmeta);
    }
    if constexpr (decltype(refill)::value && !ROPE) tile_load(t, next, 1);
    float rdot[G];
    if constexpr (ROPE) {
      float sb[2][G];
      // N^T c for one (operand block, head) at a time, the next product issued while the last one's 16 outputs are
      // folded into the score; the scheduling fences keep the compiler from hoisting all products (16 registers each)
      constexpr int NI = G * RG::NMB;
      v8h bop[2 * KK];                                      // this block's codes as fp16 B operands
      auto product = [&](int idx) {
        const int g = idx % G, mb = idx / G;
        v16f d16 = {0};
#pragma unroll
        for (int ks = 0; ks < 2 * KK; ks++)
#pragma unroll
          for (int term = 0; term < 2; term++)
            d16 = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const v8h*)&rs->img[g][mb][ks][term][lane * 8], bop[ks], d16, 0, 0, 0);
        return d16;
      };
#pragma unroll
      for (int blk = 0; blk < 2; blk++) {
        float part[G];
#pragma unroll
        for (int g = 0; g < G; g++) part[g] = 0.f;
        if constexpr (I4) {
          // int4: the lane's 8 bytes of this block are dims 16 hf .. + 15 of its token as nibble pairs (low = even dim);
          // the code minus the token's zero point is the operand (small integers: exact in fp16).  The zero point in
          // this lane's metadata belongs to token `lane` of the tile; the block's token is 32 blk + lane % 32.
          const float zb = __shfl(kz, 32 * blk + (lane & 31));
#pragma unroll
          for (int x = 0; x < 2; x++) {
            const uint32_t dw = (uint32_t)t.k[0][0][2 * blk + x];
#pragma unroll
            for (int b = 0; b < 4; b++) {
              bop[x][2 * b] = (_Float16)((float)((dw >> (8 * b)) & 15u) - zb);
              bop[x][2 * b + 1] = (_Float16)((float)((dw >> (8 * b + 4)) & 15u) - zb);
            }
          }
        } else {
        // int8 codes -> fp16 through a byte permute and one packed subtraction per two codes (codes_f16)
#pragma unroll
        for (int kk = 0; kk < KK; kk++) {
          bop[2 * kk] = __builtin_bit_cast(v8h, codes_f16(t.k[kk][blk][0], t.k[kk][blk][1]));
          bop[2 * kk + 1] = __builtin_bit_cast(v8h, codes_f16(t.k[kk][blk][2], t.k[kk][blk][3]));
        }
        }
        v16f dc = product(0);
#pragma unroll
        for (int idx = 0; idx < NI; idx++) {
          v16f dn = dc;
          if (idx + 1 < NI) dn = product(idx + 1);
          const int g = idx % G, mb = idx / G;
#pragma unroll
          for (int v = 0; v < 16; v++) {
            const int uu = 16 * mb + v;
            part[g] = fmaf(dc[v], (uu & 1) ? fs[uu >> 1] : fc[uu >> 1], part[g]);
          }
          __builtin_amdgcn_sched_barrier(0);
          dc = dn;
        }
#pragma unroll
        for (int g = 0; g < G; g++) sb[blk][g] = part[g] + __shfl_xor(part[g], 32);   // the other half wave: the other frequencies
        rope_advance(blk);                                  // to the next block of this wave: +32, then the next tile
      }
#pragma unroll
      for (int g = 0; g < G; g++) rdot[g] = lane < 32 ? sb[0][g] : sb[1][g];
    }
    if (++since_flush >= kMaxTilesPerFlush) {
      since_flush = 0;
#pragma unroll
      for (int g = 0; g < G; g++) flush(g);
    }
#pragma unroll
    for (int g = 0; g < G; g++) {
      float dot = ROPE ? rdot[g] : limbs_to_f32(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2]);
      if (I4 && !ROPE) dot = fmaf(-kz, zsum[g], dot);          // (the rotary variant has taken the zero point out of the codes)
      const float s = valid ? ksc * dot * delta[g] : -INFINITY;
      if (__builtin_amdgcn_ballot_w64(s > m[g]) != 0) {          // a new running max somewhere in this tile
        const float mn = fmaxf(m[g], wave_max(s));
        const float alpha = __builtin_amdgcn_exp2f(m[g] - mn);
        flush(g);
#pragma unroll
        for (int jj = 0; jj < KK; jj++) u[g][jj] *= alpha;
        lsum[g] *= alpha; zacc[g] *= alpha;
        m[g] = mn;
      }
      const float pw = __builtin_amdgcn_exp2f(s - m[g]);          // <= 1
      lsum[g] += pw;
      const float wt = valid ? pw * vsc : 0.f;
      if (__builtin_amdgcn_ballot_w64(wt > wref[g]) != 0) {       // a weight beyond the fixed-point range
        flush(g);
        wref[g] = 2.f * wave_max(wt);
        winv[g] = kLimbFull * __builtin_amdgcn_rcpf(wref[g]);
        omega[g] = wref[g] * (1.f / kLimbFull);
      }
      const int Q = (int)__builtin_rintf(wt * winv[g]);           // 0 .. 2^20
      // a row past the end may hold any metadata bits (NaN included): its zero point must not meet its zero weight
      if (I4) zacc[g] = fmaf((float)Q * omega[g], valid ? vz : 0.f, zacc[g]);
      wl[wave][g][0][wpos] = (uint8_t)(Q >> 14);
      wl[wave][g][1][wpos] = (uint8_t)((Q >> 7) & 127);
      wl[wave][g][2][wpos] = (uint8_t)(Q & 127);
    }
    // the wave's own LDS writes, then reads: same-wave LDS operations execute in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---------------- value pass: exact int32 accumulation, no conversion on the common path
    const v4i w0 = *(const v4i*)&wl[wave][wr_a][wr_limb][wr_g2 * 16];
    const v4i w1 = *(const v4i*)&wl[wave][wr_a][wr_limb][32 + wr_g2 * 16];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (I4) {
      const uint32_t msk = 0x0F0F0F0Fu;
      const v4i raw = t.v[0][0];
      v4i lo, hi;
#pragma unroll
      for (int x = 0; x < 4; x++) { lo[x] = raw[x] & msk; hi[x] = ((uint32_t)raw[x] >> 4) & msk; }
      vacc[0] = mfma_i8(w0, lo, vacc[0]);   // w0: limbs of even tokens, k = 16*g2 + b  <->  token 32*g2 + 2b
      vacc[0] = mfma_i8(w1, hi, vacc[0]);   // w1: limbs of odd tokens
    } else {
#pragma unroll
      for (int jj = 0; jj < KK; jj++) {
        vacc[jj] = mfma_i8(w0, t.v[jj][0], vacc[jj]);
        vacc[jj] = mfma_i8(w1, t.v[jj][1], vacc[jj]);
      }
    }
    if constexpr (decltype(refill)::value) {
      if constexpr (ROPE) tile_load(t, next, 1);      // (its key codes are read block by block)
      tile_load(t, next, 2);
    }
#ifdef WSVD_TIMELINE
    if (tl_first) { WSVD_STAMP(tl, tl_wg, wave, 4); tl_first = false; }
#endif
  };
  constexpr std::true_type kRefill{};
  constexpr std::false_type kNoRefill{};

  // ---- software pipeline over this wave's n tiles (T, T + NW, ...): compute a buffer, refill it.
  // The steady-state rounds issue their refills unconditionally, in straight-line code: a load under a branch
  // makes the compiler's wait-count bookkeeping drain the whole queue before every use, which would serialise
  // the prefetch.  Only the last rounds, where refills run out, use conditional loads.
  const int n = T < tile_end ? (tile_end - T + NW - 1) / NW : 0;
  int done = 0;
  while (done + 2 * DEPTH <= n) {
#pragma unroll
    for (int i = 0; i < DEPTH; i++) compute(kRefill, buf[i], T + (done + i) * NW, T + (done + i + DEPTH) * NW);
    done += DEPTH;
  }
  // B_V is only needed by the epilogue.  Each thread asks for the elements of its own outputs now, when the steady
  // part of the stream is over (16 latent-dim x column-pair dwords or fewer per output pass; the 8-16 KB of a head's
  // B_V are shared by many workgroups and sit in L2): they arrive behind the last tiles, so nothing waits for them.
  constexpr int BVP = STAGED ? 1 : (G * 64 * 4 + 255) / 256;     // output passes at the smallest workgroup (256 threads)
  const int half_d = p.d >> 1, hd_shift = p.d == 128 ? 6 : 5, n_pair = G * half_d, bv_items = n_pair * 4;   // d is 64 or 128
  uint32_t bvr[BVP][R / 4];
  if constexpr (!STAGED) {
    const uint32_t* bv32 = (const uint32_t*)p.BV + (size_t)cx * R * half_d;     // bf16 pairs (c, c + 1) of B_V[kv]
#pragma unroll
    for (int ps = 0; ps < BVP; ps++) {
      const int i = tid + ps * (int)blockDim.x;
      const int o = min(i >> 2, n_pair - 1), part = i & 3, c2 = o & (half_d - 1);
#pragma unroll
      for (int jj = 0; jj < R / 4; jj++) bvr[ps][jj] = bv32[(part * (R / 4) + jj) * half_d + c2];
    }
    __builtin_amdgcn_sched_barrier(0);     // the loads are issued here, not where their values are first used
  }
#pragma unroll
  for (int i = 0; i < DEPTH; i++) {
    if (done + i < n) {
      compute(kNoRefill, buf[i], T + (done + i) * NW, 0);
      if (done + i + DEPTH < n) tile_load(buf[i], T + (done + i + DEPTH) * NW, 0);
    }
  }
  done += DEPTH;
#pragma unroll
  for (int i = 0; i < DEPTH; i++)
    if (done + i < n) compute(kNoRefill, buf[i], T + (done + i) * NW, 0);

  if (FUSED) {
    // the tile with the row appended by this launch, taken by the wave whose turn it would have been
    if (own_new && wave == (new_tile - cy * chunk_tiles) % NW) {
      int budget = 1 << 16;
      while (budget > 0 && (__hip_atomic_load(p.flags + cx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.epoch ||
                            __hip_atomic_load(p.flags + p.Hkv + cx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.epoch)) {
        __builtin_amdgcn_s_sleep(16);
        budget--;
      }
      if (budget == 0 && lane == 0) atomicExch(p.err_word, (int)WSVD_E_HIP);   // never seen; keeps the kernel finite
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // drop whatever this CU / XCD cached of the tile earlier
      load_tile_coherent<R, I4>(buf[0], kplane, vplane, kmeta, vmeta, new_tile, lane);
      compute(kNoRefill, buf[0], new_tile, 0);
    }
  }
  WSVD_STAMP(tl, tl_wg, wave, 5);
  // From here on this wave only takes issue slots away from the waves of the CU that are still streaming (their next
  // tile request waits behind their arithmetic): lowest priority for the merge and the epilogue.
  __builtin_amdgcn_s_setprio(0);
  // ---- per-wave state -> workgroup merge
#pragma unroll
  for (int g = 0; g < G; g++) {
    flush(g);
    const float lw = wave_sum(lsum[g]);
    const float zc = I4 ? wave_sum(zacc[g]) : 0.f;
    if (lane == 0) { wm[g][wave] = m[g]; wls[g][wave] = lw; }
    if (lane < 32) {
#pragma unroll
      for (int jj = 0; jj < KK; jj++) wu[wave][g * R + jj * 32 + lane] = u[g][jj] - zc;
    }
  }
  WSVD_STAMP(tl, tl_wg, wave, 6);
  __syncthreads();
  WSVD_STAMP(tl, tl_wg, wave, 7);
  // The waves' (m, l, u) -> the workgroup's.  The kernel's last wave waits for this chain with nothing to overlap it,
  // so it is spread over the whole workgroup: one thread per (head, latent dim, wave slot), the slots of one (head,
  // dim) in adjacent lanes, so that each thread has one exponential and the sums over the waves are DPP reductions.
  // Slots run to the launch bound; those past the actual wave count are selected away (their LDS was never written).
  {
    constexpr int ITEMS = G * R * NWMAX;
    for (int it0 = 0; it0 < ITEMS; it0 += (int)blockDim.x) {     // uniform trip count: whole groups stay active
      const int it = it0 + tid;
      const int k = it & (NWMAX - 1), gj = min(it / NWMAX, G * R - 1);
      const int g = gj / R;
      const bool on = k < NW;
      const float mraw = wm[g][k], lraw = wls[g][k], uraw = wu[k][gj];
      const float mk = on ? mraw : -INFINITY;
      const float M = group_max<NWMAX>(mk);
      // a wave without a tile holds m = -inf, l = 0, u = 0; at least one wave of an active workgroup has rows
      const bool live = on && mk != -INFINITY;
      const float e = __builtin_amdgcn_exp2f(live ? mk - M : 0.f);
      const float U = group_sum<NWMAX>(live ? uraw * e : 0.f);
      const float L = group_sum<NWMAX>(live ? lraw * e : 0.f);
      if (k == 0 && it < ITEMS) {
        Ush[gj] = U;
        if (gj % R == 0) { Msh[g] = M; Lsh[g] = L; }
      }
    }
  }
  __syncthreads();
  WSVD_STAMP(tl, tl_wg, wave, 9);
  if constexpr (STAGED) {
    attn_tail<R, 2>(p, w, Msh, Lsh, Ush, &flag_sh, LATENT ? nullptr : (const void*)bv_lds);
  } else {
    if (!attn_merge_splits<R>(p, w, Msh, Lsh, Ush, &flag_sh)) return;
    // out[b, h, c] = sum_j (U[g][j] / L[g]) B_V[kv][j][c] with this thread's B_V elements already in registers: four
    // adjacent lanes share a column pair (a quarter of the latent dims each) and add up through DPP
#pragma unroll
    for (int ps = 0; ps < BVP; ps++) {
      const int i = tid + ps * (int)blockDim.x;
      if (ps * (int)blockDim.x < bv_items) {                      // uniform: whole quads stay active
        const int o = min(i >> 2, n_pair - 1), part = i & 3;
        const int g = o >> hd_shift, c2 = o & (half_d - 1);
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int j4 = 0; j4 < R / 4; j4 += 4) {
          const v4f u4 = *(const v4f*)&Ush[g * R + part * (R / 4) + j4];
#pragma unroll
          for (int jj = 0; jj < 4; jj++) {
            const uint32_t bb = bvr[ps][j4 + jj];
            a0 = fmaf(u4[jj], __uint_as_float(bb << 16), a0);
            a1 = fmaf(u4[jj], __uint_as_float(bb & 0xFFFF0000u), a1);
          }
        }
        WSVD_STAMP(tl, tl_wg, wave, 10);
        a0 = group_sum<4>(a0);
        a1 = group_sum<4>(a1);
        if (part == 0 && (i >> 2) < n_pair) {
          const float L = Lsh[g];
          const float rl = L > 0.f ? __builtin_amdgcn_rcpf(L) : 0.f;                 // no visible row at all: zeros
          out_put2(p, ((size_t)w.b * p.Hq + first_head(p, w.kv) + g) * p.d + 2 * c2, a0 * rl, a1 * rl);
        }
      }
    }
  }
  WSVD_STAMP(tl, tl_wg, wave, 8);
}

template <int R, int G, bool I4, int NT, bool PAGED = false>
__global__ __launch_bounds__(NT) void k_attn_mfma(AttnParams p) {
  __shared__ AttnMfmaShared<R, G, NT, false> sh;
  attn_mfma_body<R, G, I4, NT, false, 0, false, PAGED>(p, sh, blockIdx.x, blockIdx.y, blockIdx.z);
}

template <int R, int G, int NT>
__global__ __launch_bounds__(NT) void k_attn_mfma_newrow(AttnParams p) {
  __shared__ AttnMfmaShared<R, G, NT, false> sh;
  attn_mfma_body<R, G, false, NT, false, 0, false, false, true>(p, sh, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Q latent in, latent-space output out (Section 3.4: the Q latent's up-projection B_Q meets B_K^T in one small matrix
// per head, and B_V is fused into the output projection): no factor is staged at all.
template <int R, int G, bool I4, int NT>
__global__ __launch_bounds__(NT) void k_attn_mfma_latent(AttnParams p) {
  __shared__ AttnMfmaShared<R, G, NT> sh;
  attn_mfma_body<R, G, I4, NT, false, 0, true>(p, sh, blockIdx.x, blockIdx.y, blockIdx.z);
}

// ---------------------------------------------------------------- 5 to 8 query heads per kv head (I8 latents)
// One 32-token block per MFMA: all 32 rows of the A operand are in use (8 query slots x 3 limbs, slot = a + 4*h
// for row 8a + 4h + limb), so D puts the scores of queries 0..3 of token L%32 in lanes 0..31 and those of queries
// 4..7 of the same token in lanes 32..63.  Every per-query quantity (running max, weight unit, sums) is therefore a
// per-half value and the reductions run over half a wave.  The value pass has the same shape: A rows are (slot, limb)
// over the block's 32 tokens, D[slot, limb][dim] lands in the half that owns the slot.
template <int R>
struct GqaTile {
  v4i k[R / 32][2];
  v4i v[R / 32][2];
  uint32_t kmeta[2], vmeta[2];   // fp16 scales of token L%32 of block 0 / block 1
};

template <int R>
WSVD_DEV void load_gqa_tile(GqaTile<R>& t, const uint8_t* kplane, const uint8_t* vplane, const uint16_t* kmeta,
                            const uint16_t* vmeta, int tile, int lane) {
  const uint32_t off = (uint32_t)tile * (uint32_t)(64 * R) + (uint32_t)lane * 16u;
#pragma unroll
  for (int blk = 0; blk < 2; blk++)
#pragma unroll
    for (int kk = 0; kk < R / 32; kk++) {
      t.k[kk][blk] = __builtin_nontemporal_load((const v4i*)(kplane + off + (uint32_t)(blk * (32 * R) + kk * 1024)));
      t.v[kk][blk] = __builtin_nontemporal_load((const v4i*)(vplane + off + (uint32_t)(blk * (32 * R) + kk * 1024)));
    }
  const uint32_t moff = (uint32_t)tile * 64u + (uint32_t)(lane & 31);
#pragma unroll
  for (int blk = 0; blk < 2; blk++) {
    t.kmeta[blk] = __builtin_nontemporal_load(kmeta + moff + 32u * blk);
    t.vmeta[blk] = __builtin_nontemporal_load(vmeta + moff + 32u * blk);
  }
}

// LATENT: the Q latent comes in and the latent-space output goes out (no factor is read); launched with exactly NT
// threads.
// MULTI: the query slots are nq consecutive tokens x Gr heads; each slot only sees the rows up to its token's own.
// STORE: the new token's K and V latents of this launch arrive as fp32 (p.new_k / p.new_v); the workgroup whose chunk
// holds row seq_lens[b] quantises and stores them (as wsvd_latent_store would) and the attention runs over
// seq_lens[b] + 1 rows, the new row being patched into the registers of the wave that consumes its tile.  The lengths
// are advanced by the caller kernel once every workgroup of the sequence has finished.
template <int R, int NT, bool LATENT, bool MULTI, bool STORE>
WSVD_DEV void attn_gqa_body(const AttnParams& p) {
  constexpr int KK = R / 32;
  constexpr int NWMAX = NT / 64;
  constexpr int FIT = R / 16;
  constexpr int GS = 8;                 // query slots

  __shared__ v4i bv_lds[R * 128 * 2 / 16];
  __shared__ float qpart[NWMAX][32][GS];                                // per wave: partial q~ of its 32 latent dims
  __shared__ __attribute__((aligned(16))) int8_t qlimb[GS][3][R];
  __shared__ float qdelta[GS];
  __shared__ __attribute__((aligned(16))) uint8_t wl[NWMAX][GS][3][32];
  __shared__ float wm[NWMAX][GS], wls[NWMAX][GS];
  __shared__ float wu[NWMAX][GS][R];
  __shared__ float Msh[GS], Lsh[GS], Ush[GS * R];
  __shared__ __attribute__((aligned(16))) float Osh[LATENT ? 4 : GS * 128];   // un-normalised outputs of this workgroup's rows
  __shared__ int flag_sh;
  __shared__ __attribute__((aligned(16))) uint8_t new_codes[2][STORE ? R : 16];   // STORE: the row stored by this launch, K | V
  __shared__ uint16_t new_scale[2];
  __shared__ int new_ready;                                                       // STORE: set once new_codes / new_scale are written
  if (STORE && threadIdx.x == 0) new_ready = 0;                                   // (ordered before its use by the barriers below)

  const int n_raw = p.seq_lens[blockIdx.z];
  const uint32_t qs_raw = q_scale_raw(p, blockIdx.z);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NW = blockDim.x >> 6;
  const int hf = lane >> 5, l32 = lane & 31;
  const int G = p.G;
  [[maybe_unused]] long long* const tl = p.timeline;
  [[maybe_unused]] const int tl_wg = ((int)blockIdx.z * (int)gridDim.y + (int)blockIdx.y) * (int)gridDim.x + (int)blockIdx.x;
  WSVD_STAMP(tl, tl_wg, wave, 0);
  const size_t ph = (size_t)blockIdx.z * p.Hkv + blockIdx.x;
  const size_t plane_bytes = (size_t)p.t_cap * R;
  const uint8_t* kplane = p.k_codes + ph * plane_bytes;
  const uint8_t* vplane = p.v_codes + ph * plane_bytes;
  const uint16_t* kmeta = p.k_meta + ph * (size_t)p.t_cap;
  const uint16_t* vmeta = p.v_meta + ph * (size_t)p.t_cap;
  // STORE: rows attended = the old length + the row stored by this launch (a full sequence stays as it is and reports)
  const bool has_new = STORE && n_raw >= 0 && n_raw < p.t_cap;
  const int n_att = has_new ? n_raw + 1 : n_raw;
  const int chunk_tiles0 = p.chunk_rows >> 6;
  const int new_tile = n_raw >> 6;
  const bool own_new = has_new && new_tile >= (int)blockIdx.y * chunk_tiles0 && new_tile < ((int)blockIdx.y + 1) * chunk_tiles0;
  float new_c[2] = {0.f, 0.f};
  if constexpr (STORE) {
    if (n_raw >= p.t_cap && tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) atomicExch(p.err_word, (int)WSVD_E_CAPACITY);
    if (own_new && wave == NW - 1 && lane < R) {          // requested first, used after the absorption's loads are out
      new_c[0] = p.new_k[(size_t)blockIdx.z * p.new_ld + blockIdx.x * R + lane];
      new_c[1] = p.new_v[(size_t)blockIdx.z * p.new_ld + blockIdx.x * R + lane];
    }
  }

  // ---- query absorption q~ = B_K q on the matrix cores, operands straight from global memory (no staging):
  // D[j][g] = sum_c B_K[j][c] q[g][c] as V_MFMA_F32_32X32X16_BF16 with A = a 32 x 16 block of B_K (row-major, so a
  // lane's 8 operand elements are 16 contiguous bytes) and B = the queries.  An fp32 query is split into three bf16
  // terms (hi + mid + lo reproduces it to 2^-24), so the result keeps fp32 accuracy.  The (row block, 16-column step)
  // items are dealt round-robin to the waves; wave partials meet in LDS.
  constexpr int RB = R / 32;
  constexpr int MAXI = 4;                               // items per wave: RB * d/16 <= 16 items over >= 4 waves
  const int n_items = RB * (p.d >> 4);
  const int q_esz = p.q_dtype == WSVD_F32 ? 4 : p.q_dtype == WSVD_BF16 ? 2 : 1;
  const size_t q_bytes = (size_t)p.B * p.Hq * p.d * q_esz;
  const int gq = l32 < G ? l32 : 0;                     // query column of this lane (columns past G are zeroed below)
  v4i bk_raw[MAXI], q_raw[MAXI][2];
  // LATENT: q~[g][j] = sum_i c_Q[g][i] (B_Q B_K^T)[h][i][j]; work item (quarter of the i range, g, j), j fastest
  constexpr int LQ = 16;                               // rq <= 64
  constexpr int NLP = LATENT ? (4 * GS * R + NT - 1) / NT : 1;
  float lat_part[NLP];
  if constexpr (LATENT) {
    const int qn = (p.rq + 3) >> 2;
#pragma unroll
    for (int ps = 0; ps < NLP; ps++) {
      const int item = min(tid + ps * NT, 4 * G * R - 1);
      const int j = item % R, g = (item / R) % G, part = item / (R * G);
      const int h = blockIdx.x * G + g;
      const float* cq = (const float*)p.q + ((size_t)blockIdx.z * p.Hq + h) * p.rq;
      const float* fold = p.qk_fold + (size_t)h * p.rq * R + j;
      float mv[LQ], cv[LQ];
#pragma unroll
      for (int ii = 0; ii < LQ; ii++) {
        const int i = min(part * qn + ii, p.rq - 1);   // clamped: surplus slots are masked below
        mv[ii] = fold[(size_t)i * R];
        cv[ii] = cq[i];
      }
      float acc = 0.f;
#pragma unroll
      for (int ii = 0; ii < LQ; ii++) acc = (ii < qn && part * qn + ii < p.rq) ? fmaf(cv[ii], mv[ii], acc) : acc;
      lat_part[ps] = acc;
    }
  } else {
#pragma unroll
  for (int i = 0; i < MAXI; i++) {
    const int item = min(wave + i * NW, n_items - 1);   // unconditional, clamped
    const int rb = item % RB, ks = item / RB;
    bk_raw[i] = *(const v4i*)((const char*)p.BK + (((size_t)blockIdx.x * R + 32 * rb + l32) * p.d + 16 * ks + 8 * hf) * 2);
    const size_t off = (((size_t)blockIdx.z * p.Hq + (size_t)blockIdx.x * G + gq) * p.d + 16 * ks + 8 * hf) * q_esz;
    const size_t o0 = off & ~(size_t)15;
    q_raw[i][0] = *(const v4i*)((const char*)p.q + o0);
    q_raw[i][1] = *(const v4i*)((const char*)p.q + min(o0 + 16, q_bytes - 16));
  }
  }
  // ---- then the first tiles, requested speculatively below t_cap before the sequence length is known.  The barrier
  // (no memory wait) keeps every wave's small loads ahead of every wave's tile loads in the CU's memory pipeline, so
  // the absorption does not queue behind a quarter of a megabyte of tile data.
  __builtin_amdgcn_s_barrier();
  constexpr int DEPTH = 2;
  GqaTile<R> buf[DEPTH];
  const int chunk_tiles = p.chunk_rows >> 6;
  int T = (int)blockIdx.y * chunk_tiles + wave;
  // Only the first tile goes out before the absorption: a wave cannot start on q~ before it has ISSUED its tile loads,
  // and with every wave of the CU queueing two tiles that alone takes a couple of microseconds for the last one.
  const int spec_last = min(((int)blockIdx.y + 1) * chunk_tiles, p.t_cap >> 6) - 1;
  load_gqa_tile<R>(buf[0], kplane, vplane, kmeta, vmeta, min(T, spec_last), lane);
  WSVD_STAMP(tl, tl_wg, wave, 1);

  if constexpr (LATENT) {
    float* qflat = &qpart[0][0][0];                     // [4][G * R] partial sums
#pragma unroll
    for (int ps = 0; ps < NLP; ps++) {
      const int item = tid + ps * NT;
      if (item < 4 * G * R) qflat[item] = lat_part[ps];
    }
  } else {
    v16f qacc = {0};
#pragma unroll
    for (int i = 0; i < MAXI; i++) {
      if (wave + i * NW < n_items) {                    // wave-uniform
        float f[8];
        if (p.q_dtype == WSVD_F32) {
#pragma unroll
          for (int e = 0; e < 4; e++) { f[e] = __int_as_float(q_raw[i][0][e]); f[4 + e] = __int_as_float(q_raw[i][1][e]); }
        } else if (p.q_dtype == WSVD_BF16) {
#pragma unroll
          for (int e = 0; e < 4; e++) {
            f[2 * e] = __uint_as_float((uint32_t)q_raw[i][0][e] << 16);
            f[2 * e + 1] = __uint_as_float((uint32_t)q_raw[i][0][e] & 0xFFFF0000u);
          }
        } else {                                        // int8: 8 bytes, in the low or the high half of the 16 loaded
          const uint32_t d0 = (uint32_t)(hf ? q_raw[i][0][2] : q_raw[i][0][0]), d1 = (uint32_t)(hf ? q_raw[i][0][3] : q_raw[i][0][1]);
#pragma unroll
          for (int e = 0; e < 4; e++) { f[e] = (float)(int8_t)(d0 >> (8 * e)); f[4 + e] = (float)(int8_t)(d1 >> (8 * e)); }
        }
        if (l32 >= G) {
#pragma unroll
          for (int e = 0; e < 8; e++) f[e] = 0.f;
        }
        const v8bf a_op = __builtin_bit_cast(v8bf, bk_raw[i]);
        const int n_terms = p.q_dtype == WSVD_F32 ? 3 : 1;   // bf16 and int8 values are exact in one bf16 term
        for (int t3 = 0; t3 < n_terms; t3++) {
          v4i packed;
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const uint32_t h0 = __float_as_uint(f[2 * e]) & 0xFFFF0000u, h1 = __float_as_uint(f[2 * e + 1]) & 0xFFFF0000u;
            packed[e] = (int)((h0 >> 16) | h1);
            f[2 * e] -= __uint_as_float(h0);            // exact: the remainder has at most 16 significant bits
            f[2 * e + 1] -= __uint_as_float(h1);
          }
          qacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_op, __builtin_bit_cast(v8bf, packed), qacc, 0, 0, 0);
        }
      }
    }
    if (l32 < GS) {
#pragma unroll
      for (int v = 0; v < 16; v++) qpart[wave][8 * (v >> 2) + 4 * hf + (v & 3)][l32] = qacc[v];
    }
  }
  __syncthreads();
  if constexpr (STORE) {
    // every wave of this workgroup holds its copy of the old length by now (it decided own_new with it above): say so.
    // No reply is waited for.
    if (tid == 0) __hip_atomic_fetch_add(p.done + blockIdx.z, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // limbs of all 8 slots; slots past G are zero so they contribute nothing and cost nothing extra
  for (int idx = tid; idx < GS * R; idx += blockDim.x) {
    const int g = idx / R, j = idx % R;
    float v = 0.f;
    if constexpr (LATENT) {
      const float* qflat = &qpart[0][0][0];
      if (g < G) v = qflat[g * R + j] + qflat[G * R + g * R + j] + qflat[2 * G * R + g * R + j] + qflat[3 * G * R + g * R + j];
    } else {
      for (int k = (j >> 5) % RB; k < NW; k += RB) v += qpart[k][j & 31][g];   // the waves that worked on this row block
    }
    v *= p.c_scale;
    const float amax = (R == 64) ? wave_max(fabsf(v)) : half_max(fabsf(v), lane);
    const float inv = amax > 0.f ? kLimbFull / amax : 0.f;
    const int Q = (int)__builtin_rintf(v * inv);
    const int l0 = ((Q + 64) & 127) - 64;
    const int Q1 = (Q - l0) >> 7;
    const int l1 = ((Q1 + 64) & 127) - 64;
    const int l2 = (Q1 - l1) >> 7;
    qlimb[g][0][j] = (int8_t)l2;
    qlimb[g][1][j] = (int8_t)l1;
    qlimb[g][2][j] = (int8_t)l0;
    if (j == 0) qdelta[g] = amax > 0.f ? amax / kLimbFull : 0.f;
  }
  __syncthreads();
  // The second tile only now: in front of the barriers above its request blocked at the full memory pipeline, and every
  // wave of the workgroup waited there for the slowest one's request to go out (the limbs were ready 3.4 us after the
  // first tile requests).
#pragma unroll
  for (int i = 1; i < DEPTH; i++) load_gqa_tile<R>(buf[i], kplane, vplane, kmeta, vmeta, min(T + i * NW, spec_last), lane);
  if constexpr (STORE) {
    // The row, by the last wave, behind the last barrier of the prologue and so off everybody else's path (its latents were written by the
    // launch before this one, on other XCDs: they come from memory, and in front of the barrier the whole workgroup
    // waited for them); the wave that consumes the row's tile looks at new_ready when it gets there.
    if (own_new && wave == NW - 1) {                      // wave-uniform
      if (R == 64 || lane < R) {
        // the cache row for later launches (the rule and the layout of wsvd_latent_store), and a copy in LDS for this
        // one: the tile that holds the row is fetched like any other, possibly before these stores land, and the
        // wave that consumes it overwrites the row's bytes in its registers from the copy
        AppendParams ap = {};
        ap.codes[0] = const_cast<uint8_t*>(p.k_codes); ap.codes[1] = const_cast<uint8_t*>(p.v_codes);
        ap.meta[0] = const_cast<uint16_t*>(p.k_meta); ap.meta[1] = const_cast<uint16_t*>(p.v_meta);
        ap.Hkv = p.Hkv; ap.t_cap = p.t_cap; ap.latent_dtype = WSVD_I8;
#pragma unroll
        for (int pl = 0; pl < 2; pl++) {
          store_row_lanes<R>(ap, pl, (int)blockIdx.z, (int)blockIdx.x, n_raw, lane, new_c[pl]);
          const float a = lanes_max<R>(fabsf(new_c[pl]));
          uint16_t sh = 0x3C00u;
          if (a != 0.f) sh = guard_scale_f16(a / 127.0f);
          const float sc = f16_bits_to_f32(sh);
          new_codes[pl][lane] = (uint8_t)(int8_t)(int)fminf(fmaxf(__builtin_rintf(new_c[pl] / sc), -127.f), 127.f);
          if (lane == 0) new_scale[pl] = sh;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      if (lane == 0) __hip_atomic_store(&new_ready, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  }

  WSVD_STAMP(tl, tl_wg, wave, 3);
  v4i aop[KK];
  {
    const int a = l32 >> 3, hh = (l32 >> 2) & 1, limb = l32 & 3;
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      const v4i val = *(const v4i*)&qlimb[a + 4 * hh][limb < 3 ? limb : 0][kk * 32 + hf * 16];
      const v4i zero = {0, 0, 0, 0};
      aop[kk] = limb < 3 ? val : zero;
    }
  }
  const float qs = q_scale_value(p, blockIdx.z, qs_raw);
  const WorkItem w = decode_work(p, MULTI ? n_raw - p.n_after : n_att);
  if (w.n == 0) { write_zero_outputs(p, w); return; }
  if (!w.active) return;
  const int tile_end = (w.row_end + 63) >> 6;
  // MULTI: rows visible to slot a of this lane (rows [0, lim)); may be <= 0 for a token before the sequence's start
  int lim[4];
#pragma unroll
  for (int a = 0; a < 4; a++) lim[a] = MULTI ? w.n - p.nq + (a + 4 * hf) / p.Gr + 1 : 0;

  // slot a of this lane is query a + 4*hf
  float delta[4], m[4], wref[4], omega[4], winv[4], lsum[4], u[4][KK];
  v16i vacc[KK];
#pragma unroll
  for (int a = 0; a < 4; a++) {
    delta[a] = qdelta[a + 4 * hf] * qs;
    m[a] = -INFINITY; wref[a] = 0.f; omega[a] = 0.f; winv[a] = 0.f; lsum[a] = 0.f;
#pragma unroll
    for (int jj = 0; jj < KK; jj++) u[a][jj] = 0.f;
  }
#pragma unroll
  for (int jj = 0; jj < KK; jj++)
#pragma unroll
    for (int x = 0; x < 16; x++) vacc[jj][x] = 0;
  int since_flush = 0;

  auto flush = [&](int a) {
#pragma unroll
    for (int jj = 0; jj < KK; jj++) {
      u[a][jj] = fmaf(omega[a], limbs_to_f32(vacc[jj][4 * a], vacc[jj][4 * a + 1], vacc[jj][4 * a + 2]), u[a][jj]);
      vacc[jj][4 * a] = 0; vacc[jj][4 * a + 1] = 0; vacc[jj][4 * a + 2] = 0;
    }
  };

  // weights operand read position: row l32 -> slot (l32/8) + 4*((l32/4)%2), limb l32%4; k half = hf
  const int wr_q = (l32 >> 3) + 4 * ((l32 >> 2) & 1), wr_limb = min(l32 & 3, 2);

  auto compute = [&](GqaTile<R>& t, int tile) {
    if constexpr (STORE) {
      if (own_new && tile == new_tile) {                   // wave-uniform: put the row stored by this launch into the tile
        int budget = 1 << 20;                              // (written microseconds ago; the bound keeps the kernel finite)
        while (__hip_atomic_load(&new_ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0 && budget > 0) {
          __builtin_amdgcn_s_sleep(2);
          budget--;
        }
        if (budget == 0 && lane == 0) atomicExch(p.err_word, (int)WSVD_E_HIP);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int ti = n_raw & 63, blk = ti >> 5, tn = ti & 31;
#pragma unroll
        for (int b2 = 0; b2 < 2; b2++) {
          if (b2 == blk) {
#pragma unroll
            for (int kk = 0; kk < KK; kk++) {
              // K: lane (token tn, dim half hf) holds dims 32 kk + 16 hf .. + 15 of its token
              if (l32 == tn) t.k[kk][b2] = *(const v4i*)&new_codes[0][32 * kk + 16 * hf];
              // V: lane (dim 32 kk + l32, token half hf) holds 16 tokens of its dim: byte tn % 16 of the half tn / 16
              if (hf == (tn >> 4)) {
                const uint32_t byte = new_codes[1][32 * kk + l32];
                const int dw = (tn & 15) >> 2, sh8 = 8 * (tn & 3);
#pragma unroll
                for (int e = 0; e < 4; e++)
                  if (e == dw) t.v[kk][b2][e] = (int)(((uint32_t)t.v[kk][b2][e] & ~(0xFFu << sh8)) | (byte << sh8));
              }
            }
            if (l32 == tn) { t.kmeta[b2] = new_scale[0]; t.vmeta[b2] = new_scale[1]; }
          }
        }
      }
    }
    since_flush += 2;
    if (since_flush >= 2 * kMaxTilesPerFlush) {
      since_flush = 0;
#pragma unroll
      for (int a = 0; a < 4; a++) flush(a);
    }
#pragma unroll
    for (int blk = 0; blk < 2; blk++) {
      const bool valid = tile * 64 + blk * 32 + l32 < w.row_end;
      v16i acc = {0};
#pragma unroll
      for (int kk = 0; kk < KK; kk++) acc = mfma_i8(aop[kk], t.k[kk][blk], acc);
      const float ksc = f16_bits_to_f32((uint16_t)t.kmeta[blk]);
      const float vsc = f16_bits_to_f32((uint16_t)t.vmeta[blk]);
#pragma unroll
      for (int a = 0; a < 4; a++) {
        const float dot = limbs_to_f32(acc[4 * a], acc[4 * a + 1], acc[4 * a + 2]);
        const bool vis = MULTI ? (valid && tile * 64 + blk * 32 + l32 < lim[a]) : valid;
        const float s = vis ? ksc * dot * delta[a] : -INFINITY;
        if (__builtin_amdgcn_ballot_w64(s > m[a]) != 0) {          // a new running max for a query of either half
          const float mn = fmaxf(m[a], half_max(s, lane));
          // 1 in the half whose max did not move; MULTI: a half whose slot still has no visible row keeps -inf
          const float alpha = (MULTI && m[a] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m[a] - mn);
          flush(a);
#pragma unroll
          for (int jj = 0; jj < KK; jj++) u[a][jj] *= alpha;
          lsum[a] *= alpha;
          m[a] = mn;
        }
        // (a slot that has not seen a visible row yet has m = -inf: its hidden rows must not turn into NaN)
        const float pw = (MULTI && !vis) ? 0.f : __builtin_amdgcn_exp2f(s - m[a]);
        lsum[a] += pw;
        const float wt = vis ? pw * vsc : 0.f;
        if (__builtin_amdgcn_ballot_w64(wt > wref[a]) != 0) {
          flush(a);
          const float wn = 2.f * half_max(wt, lane);
          if (wn > wref[a]) {                                        // only the half that overflowed moves its unit
            wref[a] = wn;
            winv[a] = kLimbFull * __builtin_amdgcn_rcpf(wn);
            omega[a] = wn * (1.f / kLimbFull);
          }
        }
        const int Q = (int)__builtin_rintf(wt * winv[a]);
        wl[wave][a + 4 * hf][0][l32] = (uint8_t)(Q >> 14);
        wl[wave][a + 4 * hf][1][l32] = (uint8_t)((Q >> 7) & 127);
        wl[wave][a + 4 * hf][2][l32] = (uint8_t)(Q & 127);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const v4i w0 = *(const v4i*)&wl[wave][wr_q][wr_limb][hf * 16];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int jj = 0; jj < KK; jj++) vacc[jj] = mfma_i8(w0, t.v[jj][blk], vacc[jj]);
    }
  };

  const int n = T < tile_end ? (tile_end - T + NW - 1) / NW : 0;
  int done = 0;
  while (done + 2 * DEPTH <= n) {
#pragma unroll
    for (int i = 0; i < DEPTH; i++) {
      compute(buf[i], T + (done + i) * NW);
      if (done == 0 && i == 0) WSVD_STAMP(tl, tl_wg, wave, 4);
      load_gqa_tile<R>(buf[i], kplane, vplane, kmeta, vmeta, T + (done + i + DEPTH) * NW, lane);
    }
    done += DEPTH;
  }
#pragma unroll
  for (int i = 0; i < DEPTH; i++) {
    if (done + i < n) {
      compute(buf[i], T + (done + i) * NW);
      if (done + i + DEPTH < n) load_gqa_tile<R>(buf[i], kplane, vplane, kmeta, vmeta, T + (done + i + DEPTH) * NW, lane);
    }
  }
  done += DEPTH;
#pragma unroll
  for (int i = 0; i < DEPTH; i++)
    if (done + i < n) compute(buf[i], T + (done + i) * NW);

  WSVD_STAMP(tl, tl_wg, wave, 5);
  // B_V is only needed by the epilogue: requested now (it is shared by many workgroups and sits in L2), it arrives
  // while the slower waves finish
  const int fac16 = R * p.d * 2 / 16;
  StageRegs<FIT> stv;
  if constexpr (!LATENT) stage_issue<FIT>(stv, (const char*)p.BV + (size_t)blockIdx.x * R * p.d * 2, fac16);
  // per-wave state -> LDS (a wave that had no tile contributes m = -inf, l = 0, u = 0)
#pragma unroll
  for (int a = 0; a < 4; a++) {
    flush(a);
    const float lw = half_sum(lsum[a], lane);
    if (l32 == 0) { wm[wave][a + 4 * hf] = m[a]; wls[wave][a + 4 * hf] = lw; }
#pragma unroll
    for (int jj = 0; jj < KK; jj++) wu[wave][a + 4 * hf][jj * 32 + l32] = u[a][jj];
  }
  WSVD_STAMP(tl, tl_wg, wave, 6);
  if constexpr (!LATENT) stage_commit<FIT>(stv, bv_lds, fac16);
  __syncthreads();
  WSVD_STAMP(tl, tl_wg, wave, 7);
  for (int idx = tid; idx < G * R; idx += blockDim.x) {
    const int g = idx / R, j = idx % R;
    float M = wm[0][g];
    for (int k = 1; k < NW; k++) M = fmaxf(M, wm[k][g]);
    float L = 0.f, U = 0.f;
    for (int k = 0; k < NW; k++) {
      const float e = (MULTI && wm[k][g] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(wm[k][g] - M);
      L = fmaf(wls[k][g], e, L);
      U = fmaf(wu[k][g][j], e, U);
    }
    Ush[idx] = U;
    if (j == 0) { Msh[g] = M; Lsh[g] = L; }
  }
  __syncthreads();
  WSVD_STAMP(tl, tl_wg, wave, 9);
  if constexpr (LATENT) {
    attn_tail<R, 2>(p, w, Msh, Lsh, Ush, &flag_sh, nullptr);
  } else {
    // The up-projection is linear, so it is applied to this workgroup's own un-normalised accumulator BEFORE the splits
    // meet: O[g][c] = sum_j U[g][j] B_V[j][c].  The products of all splits then run side by side, and what is left for
    // the workgroup that finishes the sequence, once the other splits' words have arrived, is a weighted sum of short
    // vectors, one division and the store.  Wave g takes query slot g; lane = column pair (one LDS dword of B_V carries
    // both columns: consecutive lanes, consecutive dwords), U[g][j] is a broadcast read.
    const int half_d = p.d >> 1;
    const uint32_t* bv32 = (const uint32_t*)bv_lds;
    for (int g = wave; g < G; g += NW) {
      if (lane < half_d) {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll 8
        for (int j = 0; j < R; j++) {
          const uint32_t bb = bv32[j * half_d + lane];
          const float uj = Ush[g * R + j];
          a0 = fmaf(uj, __uint_as_float(bb << 16), a0);
          a1 = fmaf(uj, __uint_as_float(bb & 0xFFFF0000u), a1);
        }
        float2 o2; o2.x = a0; o2.y = a1;
        *(float2*)&Osh[g * p.d + 2 * lane] = o2;
      }
    }
    __syncthreads();
    WSVD_STAMP(tl, tl_wg, wave, 10);
    const bool fin = p.d == 128 ? attn_merge_splits<128>(p, w, Msh, Lsh, Osh, &flag_sh) : attn_merge_splits<64>(p, w, Msh, Lsh, Osh, &flag_sh);
    if (fin) {
      WSVD_STAMP(tl, tl_wg, wave, 11);
      for (int i = tid; i < G * p.d; i += blockDim.x) {
        const float L = Lsh[i / p.d];
        out_put(p, ((size_t)w.b * p.Hq + (size_t)w.kv * G) * p.d + i, L > 0.f ? Osh[i] / L : 0.f);   // no visible row at all: zeros
      }
    }
  }
  WSVD_STAMP(tl, tl_wg, wave, 8);
}

template <int R, int NT, bool LATENT = false, bool MULTI = false>
__global__ __launch_bounds__(NT) void k_attn_gqa(AttnParams p) {
  attn_gqa_body<R, NT, LATENT, MULTI, false>(p);
}

// latent store + attention in one launch.  The length of a sequence may advance as soon as every workgroup of the
// sequence has read the old one: each says so early in its life (a counter, no reply awaited), and one workgroup of
// the sequence waits for the count on its way out (it is complete long before; the wait is bounded, and the workgroups
// it waits for need nothing from it), clears it and writes the new length.
template <int R, int NT>
__global__ __launch_bounds__(NT) void k_attn_gqa_store(AttnParams p) {
  attn_gqa_body<R, NT, false, false, true>(p);
  // (the FIRST context chunk's workgroup: with several chunks it only delivers its partial result and is done well before
  // the chunk that merges them, so this trip to the counter is over before the launch's last workgroup is)
  if (blockIdx.x == gridDim.x - 1 && blockIdx.y == 0 && threadIdx.x == 0) {
    int* cnt = p.done + blockIdx.z;
    const int want = (int)(gridDim.x * gridDim.y);
    int budget = 1 << 16;
    while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != want && --budget > 0) __builtin_amdgcn_s_sleep(8);
    if (budget == 0) atomicExch(p.err_word, (int)WSVD_E_HIP);     // never seen; keeps the wait finite
    __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int n = p.seq_lens[blockIdx.z];
    if (n >= 0 && n < p.t_cap) p.seq_lens_rw[blockIdx.z] = n + 1;
  }
}

// Several query heads per kv head keep per-head state in registers: those instantiations are bounded to 8 waves per
// workgroup (256 registers per lane) whatever NT says, a single head may use all of NT.
template <int R, bool I4, int NT>
static hipError_t launch_m(const AttnParams& p, dim3 grid, int threads, hipStream_t s) {
  constexpr int NTG = NT > 512 ? 512 : NT;
  if (threads > (p.G == 1 ? NT : NTG) || threads % 64) return hipErrorInvalidValue;
  if (p.block_table) {                     // paged cache
    switch (p.G) {
      case 1: hipLaunchKernelGGL((k_attn_mfma<R, 1, I4, NT, true>), grid, dim3(threads), 0, s, p); break;
      case 2: hipLaunchKernelGGL((k_attn_mfma<R, 2, I4, NTG, true>), grid, dim3(threads), 0, s, p); break;
      case 3: hipLaunchKernelGGL((k_attn_mfma<R, 3, I4, NTG, true>), grid, dim3(threads), 0, s, p); break;
      case 4: hipLaunchKernelGGL((k_attn_mfma<R, 4, I4, NTG, true>), grid, dim3(threads), 0, s, p); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (p.G) {
    case 1: hipLaunchKernelGGL((k_attn_mfma<R, 1, I4, NT>), grid, dim3(threads), 0, s, p); break;
    case 2: hipLaunchKernelGGL((k_attn_mfma<R, 2, I4, NTG>), grid, dim3(threads), 0, s, p); break;
    case 3: hipLaunchKernelGGL((k_attn_mfma<R, 3, I4, NTG>), grid, dim3(threads), 0, s, p); break;
    case 4: hipLaunchKernelGGL((k_attn_mfma<R, 4, I4, NTG>), grid, dim3(threads), 0, s, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int R, int NT>
static hipError_t launch_m_newrow(const AttnParams& p, dim3 grid, int threads, hipStream_t s) {
  constexpr int NTG = NT > 512 ? 512 : NT;
  if (threads > (p.G == 1 ? NT : NTG) || threads % 64) return hipErrorInvalidValue;
  switch (p.G) {
    case 1: hipLaunchKernelGGL((k_attn_mfma_newrow<R, 1, NT>), grid, dim3(threads), 0, s, p); break;
    case 2: hipLaunchKernelGGL((k_attn_mfma_newrow<R, 2, NTG>), grid, dim3(threads), 0, s, p); break;
    case 3: hipLaunchKernelGGL((k_attn_mfma_newrow<R, 3, NTG>), grid, dim3(threads), 0, s, p); break;
    case 4: hipLaunchKernelGGL((k_attn_mfma_newrow<R, 4, NTG>), grid, dim3(threads), 0, s, p); break;
    default: return hipErrorNotSupported;
  }
  return hipGetLastError();
}
// int8 latents, rank 32 / 64, up to 4 query heads per kv head, at most 4 partial sums
hipError_t wsvd_launch_attn_newrow(const AttnParams& p, int rank, dim3 grid, int threads, hipStream_t s) {
  if (!p.pending || !p.new_k || !p.new_v || p.n_parts < 1 || p.n_parts > 4 || p.block_table) return hipErrorInvalidValue;
  if (threads < 256) return hipErrorInvalidValue;          // waves 1 and 2 carry the row's work
  if (rank == 32) return launch_m_newrow<32, 1024>(p, grid, threads, s);
  if (rank == 64) return launch_m_newrow<64, 512>(p, grid, threads, s);
  return hipErrorNotSupported;
}

template <int R, bool I4, int NT>
static hipError_t launch_m_latent(const AttnParams& p, dim3 grid, int threads, hipStream_t s) {
  if (threads > NT || threads % 64 || threads < 256) return hipErrorInvalidValue;
  switch (p.G) {
    case 1: hipLaunchKernelGGL((k_attn_mfma_latent<R, 1, I4, NT>), grid, dim3(threads), 0, s, p); break;
    case 2: hipLaunchKernelGGL((k_attn_mfma_latent<R, 2, I4, NT>), grid, dim3(threads), 0, s, p); break;
    case 3: hipLaunchKernelGGL((k_attn_mfma_latent<R, 3, I4, NT>), grid, dim3(threads), 0, s, p); break;
    case 4: hipLaunchKernelGGL((k_attn_mfma_latent<R, 4, I4, NT>), grid, dim3(threads), 0, s, p); break;
    default: return hipErrorNotSupported;
  }
  return hipGetLastError();
}

// Latent-query / latent-output attention: int8 latents with up to 8 query heads per kv head (5 to 8: exactly 512
// threads), int4 latents likewise (5 to 8: two launches over the same cache); rq <= 64.
hipError_t wsvd_launch_attn_latent(const AttnParams& p, int latent_dtype, int rank, dim3 grid, int threads, hipStream_t s) {
  if (p.rq < 1 || p.rq > 64 || !p.qk_fold) return hipErrorInvalidValue;
  if (p.G > 4 && latent_dtype == WSVD_I4 && rank == 32 && p.G <= 8) {
    // int4 latents with 5..8 query heads per kv head: two launches of the paired-block kernel, 4 heads then the rest
    AttnParams q = p;
    for (int g0 = 0; g0 < p.G; g0 += 4) {
      q.G = p.G - g0 < 4 ? p.G - g0 : 4; q.Gmem = p.G; q.g0 = g0;
      hipError_t e = launch_m_latent<32, true, 1024>(q, grid, threads > 512 ? 512 : threads, s);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  if (p.G > 4) {
    if (latent_dtype != WSVD_I8 || p.G > 8) return hipErrorNotSupported;
    if (threads != 512) return hipErrorInvalidValue;
    if (rank == 32) hipLaunchKernelGGL((k_attn_gqa<32, 512, true>), grid, dim3(512), 0, s, p);
    else if (rank == 64) hipLaunchKernelGGL((k_attn_gqa<64, 512, true>), grid, dim3(512), 0, s, p);
    else return hipErrorNotSupported;
    return hipGetLastError();
  }
  if (latent_dtype == WSVD_I8 && rank == 32) return launch_m_latent<32, false, 1024>(p, grid, threads, s);
  if (latent_dtype == WSVD_I8 && rank == 64) return launch_m_latent<64, false, 512>(p, grid, threads, s);
  if (latent_dtype == WSVD_I4 && rank == 32) return launch_m_latent<32, true, 1024>(p, grid, threads, s);
  return hipErrorNotSupported;
}

// Several query tokens per sequence, each seeing the rows up to its own: I8 latents, nq * Gr <= 8 query slots.
hipError_t wsvd_launch_attn_multi(const AttnParams& p, int rank, dim3 grid, int threads, hipStream_t s) {
  if (p.nq < 1 || p.Gr < 1 || p.nq * p.Gr != p.G || p.G > 8 || p.n_after < 0) return hipErrorInvalidValue;
  if (threads > 512 || threads % 64) return hipErrorInvalidValue;
  if (rank == 32) hipLaunchKernelGGL((k_attn_gqa<32, 512, false, true>), grid, dim3(threads), 0, s, p);
  else if (rank == 64) hipLaunchKernelGGL((k_attn_gqa<64, 512, false, true>), grid, dim3(threads), 0, s, p);
  else return hipErrorNotSupported;
  return hipGetLastError();
}

// Ranks 96 and 128 (int8 latents, one query head per kv head): the tile registers alone are 96 / 128 per lane at the
// prefetch depth of 2, so these run with at most 4 waves per workgroup and the whole 512-register file per lane.
template <int R>
static hipError_t launch_m_wide(const AttnParams& p, dim3 grid, int threads, hipStream_t s) {
  if (p.G != 1) return hipErrorNotSupported;
  if (threads > 256 || threads % 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL((k_attn_mfma<R, 1, false, 256>), grid, dim3(threads), 0, s, p);
  return hipGetLastError();
}

// latent store + attention in one launch: 5..8 query heads per kv head, I8 latents
hipError_t wsvd_launch_attn_gqa_store(const AttnParams& p, int rank, dim3 grid, int threads, hipStream_t s) {
  if (p.G <= 4 || p.G > 8) return hipErrorNotSupported;
  if (threads > 512 || threads < 256 || threads % 64) return hipErrorInvalidValue;
  if (rank == 32) hipLaunchKernelGGL((k_attn_gqa_store<32, 512>), grid, dim3(threads), 0, s, p);
  else if (rank == 64) hipLaunchKernelGGL((k_attn_gqa_store<64, 512>), grid, dim3(threads), 0, s, p);
  else return hipErrorNotSupported;
  return hipGetLastError();
}

// largest workgroup (threads) each instantiation may be launched with
// wavefronts of these kernels one CU holds at a time (register-limited): the launch policy aims at one round
int wsvd_attn_mfma_waves_per_cu(int latent_dtype, int rank, int G) {
  (void)latent_dtype;
  if (rank > 64) return 4;      // one wave per SIMD: 314 / 381 registers per lane
  return (rank == 64 || G > 1) ? 8 : 16;
}

int wsvd_attn_mfma_max_threads(int latent_dtype, int rank, int G) {
  if (rank > 64) return 256;
  if (G > 1) return 512;
  return (latent_dtype == WSVD_I8 && rank == 64) ? 512 : 1024;
}

hipError_t wsvd_launch_attn_mfma(const AttnParams& p, int latent_dtype, int rank, dim3 grid, int threads, hipStream_t s) {
  if (p.block_table && rank > 64) return hipErrorNotSupported;                   // paged cache: the paired-block kernel only
  const bool i4_32 = latent_dtype == WSVD_I4 && rank == 32;
  const bool i8_paged = p.block_table && latent_dtype == WSVD_I8 && (rank == 32 || rank == 64);
  if (p.G > 4 && p.G <= 8 && (i4_32 || i8_paged)) {
    // 5..8 query heads per kv head over int4 latents, or over a paged int8 cache: two launches of the paired-block
    // kernel, 4 heads then the rest
    AttnParams q = p;
    const int nt = threads > 512 ? 512 : threads;
    for (int g0 = 0; g0 < p.G; g0 += 4) {
      q.G = p.G - g0 < 4 ? p.G - g0 : 4; q.Gmem = p.G; q.g0 = g0;
      hipError_t e = i4_32 ? launch_m<32, true, 1024>(q, grid, nt, s)
                   : rank == 32 ? launch_m<32, false, 1024>(q, grid, nt, s) : launch_m<64, false, 512>(q, grid, nt, s);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  if (p.block_table && p.G > 4) return hipErrorNotSupported;
  if (p.G > 4) {
    // 5..8 query heads per kv head: I8 latents only
    if (latent_dtype != WSVD_I8 || p.G > 8) return hipErrorNotSupported;
    if (threads > 512 || threads < 256 || threads % 64) return hipErrorInvalidValue;
    if (rank == 32) hipLaunchKernelGGL((k_attn_gqa<32, 512>), grid, dim3(threads), 0, s, p);
    else if (rank == 64) hipLaunchKernelGGL((k_attn_gqa<64, 512>), grid, dim3(threads), 0, s, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  if (latent_dtype == WSVD_I8 && rank == 32) return launch_m<32, false, 1024>(p, grid, threads, s);
  if (latent_dtype == WSVD_I8 && rank == 64) return launch_m<64, false, 512>(p, grid, threads, s);
  if (latent_dtype == WSVD_I4 && rank == 32) return launch_m<32, true, 1024>(p, grid, threads, s);
  if (latent_dtype == WSVD_I8 && rank == 96) return launch_m_wide<96>(p, grid, threads, s);
  if (latent_dtype == WSVD_I8 && rank == 128) return launch_m_wide<128>(p, grid, threads, s);
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------- rotary variant: launch
template <int R, int G, int D, int NT, bool I4 = false>
__global__ __launch_bounds__(NT) void k_attn_rope(AttnParams p, RopeArgs ra) {
  __shared__ AttnMfmaShared<R, G, NT> sh;
  __shared__ RopeShared<R, G, D> rs;
  attn_mfma_body<R, G, I4, NT, false, D>(p, sh, blockIdx.x, blockIdx.y, blockIdx.z, &rs, &ra);
}

template <int R, int G, bool I4 = false>
static hipError_t launch_rope(const AttnParams& p, const RopeArgs& ra, dim3 grid, int threads, hipStream_t s) {
  if (p.d == 128) hipLaunchKernelGGL((k_attn_rope<R, G, 128, 512, I4>), grid, dim3(threads), 0, s, p, ra);
  else if (p.d == 64) hipLaunchKernelGGL((k_attn_rope<R, G, 64, 512, I4>), grid, dim3(threads), 0, s, p, ra);
  else return hipErrorNotSupported;
  return hipGetLastError();
}

// I8 latents (rank 32 / 64) or I4 latents (rank 32); per launch rank 32 with up to 4 query heads per kv head, rank 64 with up to 2 (the N^T operand images of all heads
// of the group live in LDS).  hipErrorNotSupported otherwise.
hipError_t wsvd_launch_attn_rope(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* q, const void* q_scale,
                                 const void* B_K, const void* B_V, const wsvd_cache& cache, int max_seq_len, double rope_base,
                                 void* out, hipStream_t s) {
  const int G = d.n_q_heads / d.n_kv_heads;
  const bool i4 = d.latent_dtype == WSVD_I4;
  if ((d.latent_dtype != WSVD_I8 && !i4) || d.factor_dtype != WSVD_BF16) return hipErrorNotSupported;
  if (d.rank != 32 && (d.rank != 64 || i4)) return hipErrorNotSupported;
  const int gmax = d.rank == 32 ? 4 : 2;               // query heads per kv head one launch holds (registers)
  AttnParams p;
  dim3 grid;
  int threads;
  // always 8 waves per workgroup: the register budget allows no more, and the N build divides its work over exactly
  // that many threads (waves without a tile of their own idle through the loop)
  wsvd_attn_plan(ctx, d, q, q_scale, B_K, B_V, cache, max_seq_len, out, p, grid, threads, 512);
  RopeArgs ra;
  const double two_pi = 6.283185307179586476925286766559;
  for (int i = 0; i < 64; i++) {
    double rev = 0.0;
    if (i < d.d_head / 2) {
      const double theta = pow(rope_base, -2.0 * i / d.d_head);
      rev = theta / two_pi;
      rev -= floor(rev);
    }
    ra.fq[i] = (uint32_t)(unsigned long long)llround(rev * 4294967296.0);    // 2^32 wraps to 0: the same angle
    // the rotations use the same rounded frequency as the start values, so that positions reached by stepping and
    // positions evaluated directly agree
    const double th = (double)ra.fq[i] / 4294967296.0 * two_pi;
    ra.rot[0][i][0] = (float)cos(th * 32.0);  ra.rot[0][i][1] = (float)sin(th * 32.0);
    ra.rot[1][i][0] = (float)cos(th * 480.0); ra.rot[1][i][1] = (float)sin(th * 480.0);
  }
  // Groups of more than gmax query heads per kv head (up to 8) run as several launches over the same cache, each on the
  // next gmax heads of every kv head: the stream is read once per launch (this variant is bound by its arithmetic per
  // (row, head), which is the same either way).
  for (int g0 = 0; g0 < G; g0 += gmax) {
    const int gl = G - g0 < gmax ? G - g0 : gmax;
    p.G = gl; p.Gmem = G; p.g0 = g0;
    hipError_t e;
    if (i4) {
      switch (gl) {
        case 1: e = launch_rope<32, 1, true>(p, ra, grid, threads, s); break;
        case 2: e = launch_rope<32, 2, true>(p, ra, grid, threads, s); break;
        case 3: e = launch_rope<32, 3, true>(p, ra, grid, threads, s); break;
        default: e = launch_rope<32, 4, true>(p, ra, grid, threads, s); break;
      }
    } else if (d.rank == 32) {
      switch (gl) {
        case 1: e = launch_rope<32, 1>(p, ra, grid, threads, s); break;
        case 2: e = launch_rope<32, 2>(p, ra, grid, threads, s); break;
        case 3: e = launch_rope<32, 3>(p, ra, grid, threads, s); break;
        default: e = launch_rope<32, 4>(p, ra, grid, threads, s); break;
      }
    } else {
      e = gl == 1 ? launch_rope<64, 1>(p, ra, grid, threads, s) : launch_rope<64, 2>(p, ra, grid, threads, s);
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---------------------------------------------------------------- fused decode step: append + attention in one launch
// The append's chain of dependent memory round trips (slice hand-off, partial sums, row store) leaves the memory
// system mostly idle; run as workgroups of the same launch as the attention it hides behind the cache stream.
// Workgroups [0, n_append) do the latent append (dispatched first, they never wait for anything), the rest the
// attention; an attention workgroup only needs the new row for the very last tile of its sequence, which it takes
// last and only after the append has published it (flags; the wait is bounded, so the kernel ends whatever happens).
// Measured on the batched int8 workload this buys nothing: with the append first the attention workgroups only get
// their slots when the append's leave (27.0 us against 26.9 us for two launches); with the two kinds interleaved the
// saturated memory system stretches every round trip of the append's chain (37 us); and the agent-scope release the
// memory model asks for before the flag (an L2 write-back) costs far more than it hides (95 us).  wsvd_decode_step
// therefore uses two launches unless the "fused_step" option asks for this kernel.  Every workgroup ends by counting itself; the last one
// advances the sequence lengths, so every reader of the old lengths is done by then.
struct StepParams {
  AttnParams a;
  AppendParams ap;
  int n_append;
  int* done;
};

template <int R, int G, int NT>
union StepShared {
  AttnMfmaShared<R, G, NT, false> attn;
  AppendMfmaShared<R, 1> app;
};

template <int R, int G, bool I4, int NT>
__global__ __launch_bounds__(NT) void k_decode_step(StepParams sp) {
  __shared__ StepShared<R, G, NT> sh;
  __shared__ int last_sh;
  const int id = blockIdx.x;
  if (id < sp.n_append) {
    append_mfma_body<R, 1>(sp.ap, sh.app, id);
  } else {
    const int r = id - sp.n_append;
    const int kv = r % sp.a.Hkv, r2 = r / sp.a.Hkv;
    attn_mfma_body<R, G, I4, NT, true>(sp.a, sh.attn, kv, r2 % sp.a.n_chunks, r2 / sp.a.n_chunks);
  }
  __syncthreads();   // every wave of this workgroup has consumed the old lengths
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(sp.done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == (int)gridDim.x - 1);
    if (last) __hip_atomic_store(sp.done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last_sh = last;
  }
  __syncthreads();
  if (!last_sh) return;
  // everything has finished: clear the row flags, so that a captured launch (whose epoch is baked into the graph) can
  // be replayed any number of times
  for (int i = threadIdx.x; i < 2 * sp.ap.Hkv; i += blockDim.x)
    __hip_atomic_store(sp.ap.flags + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int b = threadIdx.x; b < sp.ap.B; b += blockDim.x) {
    const int n = sp.ap.seq_lens[b];
    if (n >= 0 && n < sp.ap.t_cap) sp.ap.seq_lens[b] = n + 1;
    else atomicExch(sp.ap.err_word, (int)WSVD_E_CAPACITY);
  }
}

template <int R, bool I4, int NT>
static hipError_t launch_step(const StepParams& sp, int n_wg, int threads, hipStream_t s) {
  switch (sp.a.G) {
    case 1: hipLaunchKernelGGL((k_decode_step<R, 1, I4, NT>), dim3(n_wg), dim3(threads), 0, s, sp); break;
    case 2: hipLaunchKernelGGL((k_decode_step<R, 2, I4, NT>), dim3(n_wg), dim3(threads), 0, s, sp); break;
    case 3: hipLaunchKernelGGL((k_decode_step<R, 3, I4, NT>), dim3(n_wg), dim3(threads), 0, s, sp); break;
    case 4: hipLaunchKernelGGL((k_decode_step<R, 4, I4, NT>), dim3(n_wg), dim3(threads), 0, s, sp); break;
    default: return hipErrorNotSupported;
  }
  return hipGetLastError();
}

hipError_t wsvd_launch_decode_step(wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale, const void* A_K,
                                   const void* A_V, const void* q, const void* q_scale, const void* B_K, const void* B_V,
                                   const wsvd_cache& cache, int max_seq_len, void* out, hipStream_t s) {
  const bool i8 = d.latent_dtype == WSVD_I8, i4 = d.latent_dtype == WSVD_I4;
  const int G = d.n_q_heads / d.n_kv_heads;
  if (!(i8 || i4) || G > 4 || !wsvd_append_uses_mfma(d) || d.n_kv_heads > 1024 || d.batch > 32) return hipErrorNotSupported;
  if (!((i8 && (d.rank == 32 || d.rank == 64)) || (i4 && d.rank == 32))) return hipErrorNotSupported;
  StepParams sp;
  dim3 grid;
  int threads;
  // one workgroup size for both roles: the append's (its wave count follows from the d_model slice)
  const int want = wsvd_append_mfma_waves(ctx, d) * 64;
  if (want < 256 || want > wsvd_attn_mfma_max_threads(d.latent_dtype, d.rank, G)) return hipErrorNotSupported;
  wsvd_attn_plan(ctx, d, q, q_scale, B_K, B_V, cache, max_seq_len, out, sp.a, grid, threads, want);
  wsvd_append_params(ctx, d, x, x_scale, A_K, A_V, cache, sp.ap);
  if (threads != want) return hipErrorNotSupported;
  ctx->epoch = ctx->epoch == 0x7FFFFFFF ? 1 : ctx->epoch + 1;
  int* flags = (int*)ctx->ws + kWsStepFlagsInt;
  sp.a.flags = flags; sp.a.epoch = ctx->epoch; sp.a.err_word = ctx->err_word;
  sp.ap.fused = 1; sp.ap.epoch = ctx->epoch; sp.ap.flags = flags;
  sp.n_append = sp.ap.ES * sp.ap.Hkv * 2;
  sp.done = (int*)ctx->ws + kWsStepDoneInt;
  const int n_wg = sp.n_append + (int)(grid.x * grid.y * grid.z);
  if (i8 && d.rank == 32) return launch_step<32, false, 1024>(sp, n_wg, threads, s);
  if (i8 && d.rank == 64) return launch_step<64, false, 512>(sp, n_wg, threads, s);
  return launch_step<32, true, 1024>(sp, n_wg, threads, s);
}
