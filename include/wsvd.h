/*
 * wsvd.h - C ABI of the MI355X (gfx950) WSVD decode library.
 *
 * The library implements the decode-stage hot path of WSVD: single-token attention over a
 * per-head low-rank latent KV cache.  For head h the cache holds C_Kh = X A_Kh and
 * C_Vh = X A_Vh (Section 3.1 of the paper, per-head decomposition W_Kh = A_Kh B_Kh), keys and
 * values are K_h = C_Kh B_Kh, V_h = C_Vh B_Vh, and the fused decode kernel of Section 3.4
 * consumes the latent tiles in place.  Here B_Kh is folded into the query and B_Vh is applied
 * after the weighted sum of value latents, so each head's latent stream is read from HBM once.
 *
 * Conventions
 *  - Every pointer named below is a DEVICE pointer unless it says HOST.  All buffers are owned
 *    by the caller; the library allocates only in wsvd_create (one error word) and never in a
 *    hot call.  Device pointers must be 16-byte aligned.
 *  - Hot calls enqueue on the caller's HIP stream (passed as void*, NULL = default stream) and
 *    return without synchronising.  One context per stream AT A TIME: tickets, split partials and
 *    the status word live in the context's workspace, so calls on one context that overlap in time
 *    (two streams, two threads) corrupt each other.  Contexts are independent of each other.
 *  - Errors detectable on the host (NULL, unsupported shape / dtype, misalignment, workspace
 *    too small) return a non-zero status and enqueue nothing.  Conditions only the device can
 *    see (a sequence already at capacity on append) are recorded in the context's error word and
 *    reported by wsvd_check.
 *  - Head mapping for grouped-query attention: kv(h) = h / (n_q_heads / n_kv_heads).
 *  - bf16 / fp16 values are raw 16-bit patterns.
 *
 * Supported set: d_head in {64,128}; rank in {16,32,64}; n_q_heads / n_kv_heads in 1..8;
 *   latent F32  : factors, x, q F32; any rank above.
 *   latent BF16 : factors, x, q BF16.
 *   latent I8   : rank 32 or 64; factors BF16; x BF16, F32 or I8 (+fp16 scale per token); q I8 (+fp16 scale per token),
 *                 F32 or BF16.
 *                 Also rank 96 and 128 with d_head 128 and n_q_heads == n_kv_heads: wsvd_decode_attn, wsvd_decode_step,
 *                 wsvd_latent_append / wsvd_prefill_append (x BF16), wsvd_quantize_rows, cache import / export; the other
 *                 entry points return WSVD_E_UNSUPPORTED at these ranks.
 *   latent I4   : rank 32; otherwise as I8.
 *   out F32 or BF16 (round to nearest even; the decode attention entry points: wsvd_decode_attn and its _rope, _store,
 *   _paged and _static forms, wsvd_decode_step; wsvd_prefill_attn writes F32 only).  t_cap must be a multiple of 64.
 *   Any other per-head rank r (the rank sweep of Eq. 2 / Table 7: r/d = 0.9 .. 0.5) runs at the next supported rank with
 *   zero padding, which is exact: r_pad - r zero columns appended to every A_h and zero rows to every B_h give latent
 *   channels that are identically zero, change neither a row's abs-max nor any product, and quantise to code 0.
 */
#ifndef WSVD_H
#define WSVD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wsvd_ctx wsvd_ctx; /* opaque: device ordinal, error word, caller-provided workspace */

typedef enum {
  WSVD_OK = 0,
  WSVD_E_NULL = 1,        /* a required pointer is NULL */
  WSVD_E_SHAPE = 2,       /* a size is out of the supported set or inconsistent */
  WSVD_E_DTYPE = 3,       /* dtype combination not supported */
  WSVD_E_ALIGN = 4,       /* a device pointer is not 16-byte aligned */
  WSVD_E_CAPACITY = 5,    /* a sequence was at t_cap on append (device-detected), or max_seq_len > t_cap */
  WSVD_E_UNSUPPORTED = 6, /* valid request this build does not implement */
  WSVD_E_HIP = 7,         /* a HIP runtime call failed */
  WSVD_E_WORKSPACE = 8    /* workspace missing or too small */
} wsvd_status;

typedef enum { WSVD_F32 = 0, WSVD_BF16 = 1, WSVD_F16 = 2, WSVD_I8 = 3, WSVD_I4 = 4 } wsvd_dtype;

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, d_head, d_model, rank; /* rank = r_K = r_V (uniform per-head rank) */
  int32_t t_cap;        /* rows of capacity per (sequence, kv head); multiple of 64 */
  int32_t latent_dtype; /* F32 | BF16 | I8 (symmetric, fp16 scale per row) | I4 (asymmetric, fp16 scale + zero point per row) */
  int32_t factor_dtype; /* dtype of A_K, A_V, B_K, B_V */
  int32_t x_dtype;      /* dtype of the hidden state given to wsvd_latent_append */
  int32_t q_dtype;      /* dtype of the query given to wsvd_decode_attn; I8 carries one fp16 scale per token */
  int32_t out_dtype;    /* F32 */
  float sm_scale;       /* softmax scale; 0 means 1/sqrt(d_head) */
} wsvd_layer_desc;

/*
 * The latent cache (Section 3.1: C_Kh, C_Vh of shape L x r per head), one K plane and one V plane.
 * Logical content: row t of kv head h of sequence b, t < seq_lens[b].
 *
 * DEVICE layout of the code planes.  F32 / BF16: row-major [B, Hkv, t_cap, rank].
 * I8 / I4: each block of tokens is stored as the register image of the gfx950 MFMA operand it
 * feeds, so a wavefront's 64 x 16-byte load IS the operand (no unpack, no shuffle):
 *   I8, K plane: per (b,h) blocks of 32 tokens, rank*32 bytes each; byte of (token n, dim j) at
 *        ((j/32*2 + (j%32)/16)*32 + n)*16 + j%16
 *   I8, V plane: same block size; byte of (token n, dim j) at
 *        ((j/32*2 + n/16)*32 + j%32)*16 + n%16          (token-minor: the contraction runs over tokens)
 *   I4 (rank 32), K plane: blocks of 64 tokens, 1024 bytes; token tt = slot*32 + n, dims (j, j+1) share a byte:
 *        (j/16)*512 + n*16 + slot*8 + (j%16)/2, low nibble = even j
 *   I4, V plane: blocks of 64 tokens; tokens (tt, tt+1) share a byte:
 *        ((tt/32)*32 + j)*16 + (tt%32)/2, low nibble = even tt
 * Callers never need these formulas: wsvd_cache_import / wsvd_cache_export convert from / to the
 * plain row-major ("logical") format in which wsvd_quantize_rows writes.
 * Metadata planes: I8: fp16 scale [B,Hkv,t_cap]; I4: {fp16 scale, fp16 zero point} [B,Hkv,t_cap][2];
 * F32/BF16: unused (may be NULL).
 */
typedef struct {
  void *k_codes, *v_codes;
  void *k_meta, *v_meta;
  int32_t *seq_lens; /* [B] valid rows per sequence; wsvd_latent_append increments it on the device */
} wsvd_cache;

/* Create / destroy a context bound to a device ordinal.  Allocates a 4-byte device error word. */
wsvd_status wsvd_create(wsvd_ctx **out, int device_ordinal);
wsvd_status wsvd_destroy(wsvd_ctx *ctx);

/* Bytes of ONE code plane and ONE metadata plane (K or V) for this layer (HOST outputs). */
wsvd_status wsvd_cache_bytes(const wsvd_layer_desc *desc, size_t *codes_bytes, size_t *meta_bytes);

/* Scratch the hot calls need for this layer (counters, the words workgroups hand partial results over in); HOST output. */
wsvd_status wsvd_workspace_bytes(const wsvd_layer_desc *desc, size_t *bytes);

/* Hand the context a caller-owned device scratch buffer.  Clears it (synchronously). */
wsvd_status wsvd_set_workspace(wsvd_ctx *ctx, void *dev_ptr, size_t bytes);

/*
 * Down-projection factors are constants of the layer; the append kernels read them in a matrix-core friendly
 * packing: blocks of 32 latent channels x 16 model dims stored as the 64-lane x 16-byte register image of a
 * 32x32x16 MFMA operand (channels padded to a multiple of 32).  wsvd_pack_factor_a converts, once, from the
 * paper's shape A_h in R^{E x r} (Section 3.1), given row-major as [Hkv, d_model, rank] of factor_dtype.
 * Both pointers are device pointers; A_packed must hold wsvd_factor_a_bytes bytes.
 */
wsvd_status wsvd_factor_a_bytes(const wsvd_layer_desc *desc, size_t *bytes);
wsvd_status wsvd_pack_factor_a(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *A_row_major, void *A_packed,
                               void *hip_stream);

/*
 * Decode-step cache update (Section 3.4, decoding pipeline: the new token is down-projected per head
 * and its K and V latents are stored in the cache).  For every sequence b and kv head h:
 *   c_K = x[b,:] A_K[h], c_V = x[b,:] A_V[h]  (fp32 accumulation), rounded to latent_dtype
 *   (I8 / I4: the quantiser documented at wsvd_quantize_rows), written at row seq_lens[b];
 * then seq_lens[b] += 1.  A sequence with seq_lens[b] >= t_cap is left unchanged and the
 * context's error word is set to WSVD_E_CAPACITY.
 *   x       [B, d_model] of x_dtype.
 *   x_scale x_dtype I8 (quantised latents only): fp16 [B], one scale per token; the hidden state is x * x_scale (the
 *           activation format of Section 4.2).  NULL otherwise.  The matrix-core kernels, the paged cache, the tiled
 *           prefill and the single-launch step take BF16 hidden states; I8 and F32 ones go through the vector-ALU
 *           append kernel (functional path).  With int4 weights as well, wsvd_linear_w4a8_split + wsvd_latent_store
 *           is the route.
 *   A_K,A_V PACKED by wsvd_pack_factor_a (wsvd_factor_a_bytes bytes each).  d_model must be a multiple of 64.
 */
wsvd_status wsvd_latent_append(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *x, const void *x_scale,
                               const void *A_K, const void *A_V, wsvd_cache *cache, void *hip_stream);

/*
 * The store half of the cache update for callers that compute the new token's latents with their own GEMM
 * (the quantised setting of Section 4.2, where the down-projection is an int4-weight / int8-activation matmul
 * fused with the query projection: see wsvd_linear_w4a8).  For every sequence b and kv head h the fp32 row
 *   c_K[b*ld + h*rank .. + rank),  c_V[b*ld + h*rank .. + rank)        (DEVICE pointers, ld in floats)
 * is rounded to latent_dtype exactly as wsvd_latent_append would and written at row seq_lens[b]; then
 * seq_lens[b] += 1.  Capacity handling as in wsvd_latent_append.  c_K and c_V may point into one buffer.
 */
wsvd_status wsvd_latent_store(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const float *c_K, const float *c_V,
                              int64_t ld, wsvd_cache *cache, void *hip_stream);

/*
 * Decode attention over the latent cache (Section 3.4 fused kernel; Section 2.4 flash-decoding
 * schedule: sequence tiles, online softmax, parallel sequence splits merged at the end).
 * For every b and query head h with kv = kv(h), n = seq_lens[b]:
 *   out[b,h,:] = softmax_t( sm_scale * q[b,h,:] . (C_K[b,kv,t,:] B_K[kv]) ) . (C_V[b,kv,:,:] B_V[kv])
 * over rows t < n; n == 0 gives zeros.  Computed as q~ = B_K q, scores on the latent rows, u = p^T C_V,
 * out = u B_V (associativity only).
 *   q [B,Hq,d_head] of q_dtype; q_scale fp16 [B] iff q_dtype == I8 (buffer padded to a multiple of 4 bytes)
 *   B_K,B_V [Hkv, rank, d_head] of factor_dtype;  out [B,Hq,d_head] F32
 *   max_seq_len: HOST upper bound on seq_lens (sizes the grid); must be <= t_cap.  A sequence found to be longer
 *                than the rows the grid covers (max_seq_len rounded up to whole chunks) sets the device status word
 *                to WSVD_E_SHAPE (wsvd_check); its output is then computed from the covered rows only.
 */
wsvd_status wsvd_decode_attn(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *q, const void *q_scale,
                             const void *B_K, const void *B_V, const wsvd_cache *cache, int32_t max_seq_len,
                             void *out, void *hip_stream);

/*
 * wsvd_latent_store followed by wsvd_decode_attn (Section 3.4, decoding pipeline: store the new token's latents, then
 * attend over the cache including them) as ONE call: c_K, c_V, ld as for wsvd_latent_store; q, q_scale, B_K, B_V, out
 * as for wsvd_decode_attn; max_seq_len bounds the lengths AFTER the store (>= 1).  Results are those of the two calls.
 * With I8 latents and 5 to 8 query heads per kv head it is a single launch: the workgroup whose context chunk holds
 * the new row quantises and stores it, keeps a copy for the wavefront that consumes the row's tile, and the last
 * workgroup of a sequence to finish advances its length; every other combination runs the two kernels back to back.
 * A sequence already at t_cap is left unchanged, is attended over its t_cap rows, and WSVD_E_CAPACITY is recorded in
 * the device status word.
 */
wsvd_status wsvd_decode_attn_store(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const float *c_K, const float *c_V, int64_t ld,
                                   const void *q, const void *q_scale, const void *B_K, const void *B_V,
                                   wsvd_cache *cache, int32_t max_seq_len, void *out, void *hip_stream);

/*
 * Paged cache (serving systems hand out the cache in pages): the K / V code and metadata planes are POOLS of n_pages
 * pages; a page holds page_rows consecutive rows (a multiple of 64) of EVERY kv head of one sequence, each in the
 * device layout of the contiguous planes (page p, kv head h: page_rows * row_bytes code bytes at
 * ((p * Hkv + h) * page_rows * row_bytes, metadata likewise); block_table[b][i] names the page with rows
 * [i * page_rows, (i + 1) * page_rows) of sequence b.  desc->t_cap must equal max_pages * page_rows.  Entries for pages
 * a sequence does not reach yet are not read for results; an append into a row whose entry is outside [0, n_pages)
 * stores nothing and records WSVD_E_SHAPE in the device status word.  The caller owns pools and table.
 * Quantised latents (I8, I4), rank <= 64, up to 8 query heads per kv head; x and factors BF16 for the append
 * (WSVD_E_UNSUPPORTED otherwise).  Results are those of wsvd_latent_append / wsvd_decode_attn on the same rows (bit for
 * bit up to 4 query heads per kv head and for I4; 5..8 heads over I8 latents run as two launches over head sets of 4,
 * the cache read by each, and agree with wsvd_decode_attn to fp32 rounding).
 */
typedef struct {
  void *k_codes, *v_codes;       /* DEVICE pools */
  void *k_meta, *v_meta;
  int32_t *seq_lens;             /* DEVICE [B] */
  const int32_t *block_table;    /* DEVICE [B][max_pages] */
  int32_t page_rows, max_pages, n_pages;
} wsvd_paged_cache;
/* Bytes of ONE code pool and ONE metadata pool (K or V) of n_pages pages (HOST outputs). */
wsvd_status wsvd_paged_cache_bytes(const wsvd_layer_desc *desc, int32_t page_rows, int32_t n_pages, size_t *codes_bytes,
                                   size_t *meta_bytes);
wsvd_status wsvd_latent_append_paged(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *x, const void *x_scale,
                                     const void *A_K, const void *A_V, wsvd_paged_cache *cache, void *hip_stream);
/* Prompt into a paged cache: wsvd_prefill_append (its tiled projection: any number of tokens, one sequence or all with
 * seq_index = -1, x [n_seq, n_tokens, d_model] BF16, int4 latents from an even length) with the rows going to the pages
 * of block_table; a table entry outside the pools is reported (WSVD_E_SHAPE through wsvd_check) and its rows are not
 * stored.  The stored bytes are those wsvd_prefill_append puts into a contiguous cache. */
wsvd_status wsvd_prefill_append_paged(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *x, int32_t n_tokens,
                                      int32_t seq_index, const void *A_K, const void *A_V, wsvd_paged_cache *cache,
                                      void *hip_stream);
/* Attention over the prompt from a paged cache: wsvd_prefill_attn's tiled kernel (any n_q; BF16 queries, I8 latents,
 * F32 out) with every 32-token cache block taken from the page the table names.  Results are those of
 * wsvd_prefill_attn (tiled kernel) on the same rows. */
wsvd_status wsvd_prefill_attn_paged(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *q, int32_t n_q, int32_t n_after,
                                    const void *B_K, const void *B_V, const wsvd_paged_cache *cache, int32_t max_seq_len,
                                    void *out, void *hip_stream);
wsvd_status wsvd_decode_attn_paged(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *q, const void *q_scale,
                                   const void *B_K, const void *B_V, const wsvd_paged_cache *cache, int32_t max_seq_len,
                                   void *out, void *hip_stream);

/*
 * wsvd_decode_attn for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results as
 * wsvd_decode_attn, but the words through which the splits of a long sequence reach the workgroup that merges them
 * live in an array that is part of the library image (8 MiB of device memory per GPU the library runs on, held until
 * the process ends) instead of the workspace set with wsvd_set_workspace, which is neither needed nor touched.  The
 * call allocates nothing and frees nothing.
 *   Limit: 65536 + 8 * batch * n_q_heads * n_chunks * (max(rank, d_head) + 2) bytes must fit in the 8 MiB, n_chunks being the
 *   number of context splits the launch policy picks for this call (1 when batch * n_kv_heads alone fills the chip:
 *   then the term is 0; at most ceil(max_seq_len / 256)); all five documented workloads fit; WSVD_E_WORKSPACE
 *   otherwise, nothing enqueued.
 *   Every call on a GPU shares that GPU's array, from every context and stream: calls that overlap in time on one
 *   GPU race on it.  Calls on one stream are ordered and safe.
 * Enqueues the attention kernel on hip_stream, behind a small clearing kernel when the context is split; error
 * behaviour as wsvd_decode_attn.
 */
wsvd_status wsvd_decode_attn_static(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *q, const void *q_scale,
                                    const void *B_K, const void *B_V, const wsvd_cache *cache, int32_t max_seq_len,
                                    void *out, void *hip_stream);

/*
 * Tuning of ONE context's work decomposition; correct use never needs it, results agree to fp32 rounding whatever is
 * set.  The setting applies to the calls made on this context afterwards (two contexts may differ).
 *   "wg_per_cu":   scales the number of wavefronts the attention grid aims for (default 4 = one resident round)
 *   "min_chunk":   smallest context chunk per attention workgroup in rows: 0 (default) = automatic (256 rows, and no
 *                  split of a (sequence, kv head) whose latents are too few for a split to pay); else a multiple of 64
 *                  (values below 256 count as 256), taken as given
 *   "max_threads": cap on the attention workgroup size (0 = the kernel's own bound; else 256, 512, 768 or 1024)
 *   "append_mode": 0 = the default append kernel; n > 0 = the kernel that cuts d_model into n equal slices
 * Unknown names and values out of range return WSVD_E_SHAPE.  (Names that switch between alternative kernels for
 * tests are listed in wsvd_test.h.)
 */
wsvd_status wsvd_ctx_set_option(wsvd_ctx *ctx, const char *name, int value);

/*
 * Decode attention for a backbone with rotary position embedding: the kernel of Section 3.4 taken literally.
 * The key tile K = C_K B_K is formed on chip, key t is rotated by its position t (its row index), the query by the
 * position of the newest row, seq_lens[b] - 1, and the rotated product q_rot . K_rot[t] replaces q . K[t]; everything
 * else is wsvd_decode_attn.  Rotation: dims (i, i + d_head/2) form a plane turned by position * theta_i with
 * theta_i = rope_base^(-2i/d_head) ("rotate-half" pairing).  With the rotation between the reconstruction and the
 * product, B_K cannot be folded into the query, so every cached row costs 2 * rank * d_head flops per query head.
 * Supported: I8 latents (rank 32 or 64) and I4 latents (rank 32; the codes minus the token's zero point are the
 * operands), bf16 factors, up to 8 query heads per kv head (one launch holds 4 heads of a
 * group at rank 32 and 2 at rank 64; larger groups run as several launches over the same cache, one per set of
 * heads); WSVD_E_UNSUPPORTED otherwise.  rope_base > 1 (10000 is the usual value).
 */
wsvd_status wsvd_decode_attn_rope(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *q, const void *q_scale,
                                  const void *B_K, const void *B_V, const wsvd_cache *cache, int32_t max_seq_len,
                                  float rope_base, void *out, void *hip_stream);

/*
 * One decode step of a layer (Section 3.4, decoding pipeline): wsvd_latent_append followed by wsvd_decode_attn,
 * with the same arguments and the same results (the attention includes the row just appended).  Two launches.
 * I8 latents, rank 32 / 64, bf16 hidden states and factors, at most 4 query heads per kv head: the first launch only
 * projects (partial sums over slices of d_model into the workspace) and advances the lengths; the attention launch
 * sums the slices, quantises, stores the new rows and takes them from registers, so the hand-off between the
 * append's workgroups is the kernel boundary itself ("step_deferred" setting of wsvd_test.h; the stored codes may
 * differ from wsvd_latent_append's where the fp32 sums, taken in another order, fall on the other side of a rounding
 * boundary).  Every other combination: the append kernel and the attention kernel back to back.  A single-launch
 * kernel also exists ("fused_step" setting); it measured no faster on MI355X, so it is not the default.
 *   max_seq_len: host upper bound on the sequence lengths AFTER the append (>= 1).
 * Capacity handling as in wsvd_latent_append: a full sequence is attended as it is and reported by wsvd_check.
 */
wsvd_status wsvd_decode_step(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *x, const void *x_scale,
                             const void *A_K, const void *A_V, const void *q, const void *q_scale, const void *B_K,
                             const void *B_V, wsvd_cache *cache, int32_t max_seq_len, void *out, void *hip_stream);

/* Synchronise the stream and return (then clear) the device-side error word. */
wsvd_status wsvd_check(wsvd_ctx *ctx, void *hip_stream);

const char *wsvd_status_str(wsvd_status s);

/*
 * Quantise fp32 latent rows into the LOGICAL row-major format (the same device routine the append
 * uses).  Per-token-per-head granularity after the per-token symmetric activation quantisation of
 * Section 4.2; rounding rules (IEEE fp32, round-to-nearest-even, true division):
 *   I8: a = max|c_j|; a == 0 -> scale 1, codes 0; else s = fp16(a/127) (0 -> 2^-24, inf -> 65504),
 *       code_j = clamp(rint(c_j / float(s)), -127, 127).
 *   I4: lo = min(min c, 0), hi = max(max c, 0); hi == lo -> s = 1, z = 0, codes 0; else
 *       s = fp16((hi-lo)/15) (same guards), z = clamp(rint(-lo/float(s)), 0, 15),
 *       code_j = clamp(int(rint(c_j/float(s))) + int(z), 0, 15); element 2i in the low nibble of byte i.
 *   c [n_rows, rank] fp32 -> codes [n_rows, rank] int8 or [n_rows, rank/2] bytes;
 *   meta: fp16 [n_rows] (I8) or {scale, zero point} fp16 [n_rows][2] (I4).
 */
wsvd_status wsvd_quantize_rows(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const float *c, int64_t n_rows,
                               void *codes, void *meta, void *hip_stream);

/*
 * Copy rows [t0, t0+n_rows) of every (b, kv head) between the logical row-major format
 * ([B,Hkv,n_rows,row_bytes] codes, [B,Hkv,n_rows(,2)] metadata) and the device layout of one plane.
 * which_plane: 0 = K, 1 = V.  Bit-preserving.  Does not touch seq_lens.
 */
wsvd_status wsvd_cache_import(wsvd_ctx *ctx, const wsvd_layer_desc *desc, int32_t which_plane, const void *codes,
                              const void *meta, int32_t t0, int32_t n_rows, wsvd_cache *cache, void *hip_stream);
wsvd_status wsvd_cache_export(wsvd_ctx *ctx, const wsvd_layer_desc *desc, int32_t which_plane,
                              const wsvd_cache *cache, int32_t t0, int32_t n_rows, void *codes, void *meta,
                              void *hip_stream);

/*
 * Prefill of the cache (Section 3.4: during prefilling the input sequence is projected into low-rank latents and the K, V
 * latents are stored as the cache): x [n_tokens, E] holds consecutive tokens of ONE sequence, seq_index; token i is
 * projected like wsvd_latent_append's rows, stored at row seq_lens[seq_index] + i of every kv head, and the length
 * advances by n_tokens.  x, x_scale, A_K, A_V as for wsvd_latent_append.  Up to 64 tokens per call for every
 * supported format (the append kernels; the workspace must be large enough for a descriptor whose batch is n_tokens,
 * WSVD_E_WORKSPACE otherwise); any number of tokens per call with I8 latents and BF16 hidden states and factors (a tiled
 * projection on the matrix cores, no workspace; WSVD_E_SHAPE for n_tokens > 64 with other formats).  With those formats
 * seq_index = -1 stores n_tokens rows for EVERY sequence of the batch in one launch: x is then [batch, n_tokens, d_model]
 * and each sequence's rows start at its own length (WSVD_E_SHAPE for seq_index = -1 with other formats).  Rows beyond
 * t_cap are not stored: the sequence is left full and WSVD_E_CAPACITY is recorded in the device status word.  F32, BF16,
 * I8 and I4 latents.  I4 (x and factors BF16, any n_tokens, one sequence or all): a value byte holds two consecutive
 * rows, so every target sequence must stand at an EVEN length when the call is made (a fresh prompt does); a sequence at
 * an odd length is left unchanged and WSVD_E_SHAPE is recorded in the device status word.  Attention over the prompt
 * itself is not part of this call.
 */
wsvd_status wsvd_prefill_append(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *x, const void *x_scale,
                                int32_t n_tokens, int32_t seq_index, const void *A_K, const void *A_V, wsvd_cache *cache,
                                void *hip_stream);

/*
 * Attention of several consecutive query tokens per sequence, each seeing the cache rows up to and including its own
 * (the attention of prefilling, Section 3.4, in chunks; also multi-token decoding).  The n_q tokens' latents are already
 * in the cache (wsvd_prefill_append), followed by n_after later rows: query token i of sequence b sits at row
 * seq_lens[b] - n_after - n_q + i.  A token whose row index is negative, and every token of an empty sequence, gets
 * zeros.
 *   q and out: [B, Hkv, n_q, G, d] (kv head, then token, then the G = Hq / Hkv query heads of that kv head), q of
 *   desc->q_dtype (F32 or BF16; WSVD_E_DTYPE for I8), out F32.  I8 latents, BF16 factors (WSVD_E_UNSUPPORTED otherwise).
 *   n_q * G <= 8: the decode kernel with one query slot per (token, head); the workspace must be large enough for a
 *   descriptor with Hkv * n_q * G query heads (WSVD_E_WORKSPACE otherwise).  n_q * G > 8: a tiled kernel, BF16 queries
 *   only (WSVD_E_UNSUPPORTED for F32), no workspace, any n_q (a whole prompt in one call); max_seq_len is not used by it.
 *   Its value product runs on fp16 operands (code * scale and the softmax weights, each rounded to 2^-12 relative):
 *   outputs agree with the exact result to about 2e-4 relative, the slot kernel's to about 1e-5.
 *   Stream, pointer and error conventions as wsvd_decode_attn.
 */
wsvd_status wsvd_prefill_attn(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *q, int32_t n_q, int32_t n_after,
                              const void *B_K, const void *B_V, const wsvd_cache *cache, int32_t max_seq_len, void *out,
                              void *hip_stream);

/*
 * Decode attention of the conventional whole-matrix scheme the per-head method is contrasted with (Section 3.1 and panel
 * (b) of its figure; the "W/o per-head" variant of the latency appendix): ONE latent of rank R per token and plane,
 * C_K = X A_K, shared by all heads; head h has its own up-projections B_Kh, B_Vh [R, d]:
 *     K_h = C_K B_Kh,  V_h = C_V B_Vh,  o_h = softmax(sm_scale * q_h K_h^T) V_h       (sm_scale <= 0: 1 / sqrt(d_head)).
 * The kernels absorb B_Kh into the query and B_Vh into the output, and run all heads as the columns of one product over
 * the shared latent, which is therefore streamed once per step (not once per head).
 *   n_heads = 32; d_head 64 or 128; rank 256, 512 or 1024, or a multiple of 128 up to 4096 (these with t_cap <= 16384:
 *   one more small launch, the latent walked in slabs of 1024 dims); t_cap a multiple of 128 (WSVD_E_UNSUPPORTED /
 *   WSVD_E_SHAPE).
 *   q [B, H, d] BF16, B_K and B_V [H, R, d] BF16, out [B, H, d] F32 (all DEVICE, 16-byte aligned).
 *   k_codes, v_codes: int8 latents, one plane of t_cap * R bytes per sequence, in 32-token blocks of 32 * R bytes.  Byte
 *   of (token t, dim j): K plane  (t / 32) * 32 R + (((j / 32) * 2 + (j % 32) / 16) * 32 + t % 32) * 16 + j % 16,
 *                        V plane  (t / 32) * 32 R + (((j / 32) * 2 + (t % 32) / 16) * 32 + j % 32) * 16 + t % 16
 *   (the per-head cache layout with a single head of rank R).  k_scale, v_scale [B, t_cap] fp16: one symmetric scale per
 *   token and plane (value = code * scale).  seq_lens [B] int32 (DEVICE): rows [0, seq_lens[b]) are attended; a sequence
 *   with no rows gets zeros; rows beyond may hold anything.
 *   workspace (DEVICE, 16-byte aligned) of at least wsvd_shared_workspace_bytes(...) bytes, owned by the caller, free for
 *   reuse when the stream has passed the call (WSVD_E_WORKSPACE when too small).  Three launches on hip_stream; no host
 *   synchronisation.  Scores run on exact int8 products (the query as three 7-bit limbs); the value product on fp16
 *   operands (2^-12 relative): outputs agree with the exact result to about 2e-4 relative.
 */
wsvd_status wsvd_shared_workspace_bytes(int32_t batch, int32_t n_heads, int32_t d_head, int32_t rank, int32_t t_cap, size_t *bytes);
wsvd_status wsvd_decode_attn_shared(wsvd_ctx *ctx, int32_t batch, int32_t n_heads, int32_t d_head, int32_t rank, int32_t t_cap,
                                    float sm_scale, const void *q, const void *B_K, const void *B_V, const void *k_codes,
                                    const void *v_codes, const void *k_scale, const void *v_scale, const int32_t *seq_lens,
                                    void *workspace, size_t workspace_bytes, void *out, void *hip_stream);

/*
 * The rest of the decoding pipeline (Section 3.4, decoding-pipeline figure): the query is per-head low-rank too, and
 * the V-path up-projection is fused into the output projection.
 *
 * wsvd_fold_qk: M_h = B_Q,h B_K,kv(h)^T, so that q_h K^T = (c_Q,h M_h) C_K^T.  Set-up, once per model.
 *   B_Q [Hq, rq, d] and B_K [Hkv, r, d] of desc->factor_dtype (DEVICE); out [Hq, rq, r] F32 (DEVICE).  1 <= rq <= 64.
 * wsvd_fold_vo: W'_O[:, h r + j] = sum_c B_V,kv(h)[j, c] W_O[:, h d + c], so that W_O o = W'_O u with u the latent-space
 *   attention output.  Set-up, once per model.  B_V [Hkv, r, d] of desc->factor_dtype; W_O [E, Hq d] F32, one row per
 *   output channel; out [E, Hq r] F32.  All DEVICE pointers.
 * wsvd_decode_attn_latent: the attention that goes with the two folds.  c_Q [B, Hq, rq] F32 is the Q latent as it leaves
 *   its down-projection, qk_fold the output of wsvd_fold_qk; scores sm_scale * C_K (c_Q M)^T, softmax, and
 *   u_out[b, h, :] = p^T C_V [B, Hq, r] F32 (zeros for an empty sequence).  B_K and B_V are not read.
 *   I8 or I4 latents, rank up to 64, at most 8 query heads per kv head (WSVD_E_UNSUPPORTED otherwise);
 *   desc->q_dtype is ignored.
 *   Pointers DEVICE, 16-byte aligned; max_seq_len, workspace, stream and error behaviour as wsvd_decode_attn.
 */
wsvd_status wsvd_fold_qk(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *B_Q, int32_t rq, const void *B_K, void *out,
                         void *hip_stream);
wsvd_status wsvd_fold_vo(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *B_V, const void *W_O, void *out,
                         void *hip_stream);
wsvd_status wsvd_decode_attn_latent(wsvd_ctx *ctx, const wsvd_layer_desc *desc, const void *c_Q, int32_t rq,
                                    const void *qk_fold, const wsvd_cache *cache, int32_t max_seq_len, void *u_out,
                                    void *hip_stream);

/*
 * Row kernels of a pre-norm decoder layer in the quantised setting of Section 4.2 (activations per-token symmetric
 * int8, same rounding rules as wsvd_quantize_act_i8).  rows <= any, cols / F multiples of 4 and <= 16384; DEVICE
 * pointers, 16-byte aligned.
 * wsvd_rmsnorm_quant_i8: r = x (+ y_add); if y_add is given the sum is written to x_out [rows, cols] F32 (the
 *   residual stream; x_out may alias x); h = r / sqrt(mean(r^2) + eps) * gain; h -> codes int8 [rows, cols], scale fp16
 *   [rows].  x, y_add [rows, cols] F32, gain [cols] F32.
 * wsvd_swiglu_quant_i8: gate_up [rows, 2F] F32 with the gate in columns [0, F) and the up branch in [F, 2F);
 *   a = silu(gate) * up -> codes int8 [rows, F], scale fp16 [rows].
 */
wsvd_status wsvd_rmsnorm_quant_i8(wsvd_ctx *ctx, const void *x, const void *y_add, const void *gain, float eps, int64_t rows,
                                  int64_t cols, void *x_out, int8_t *codes, void *scale_f16, void *hip_stream);
wsvd_status wsvd_swiglu_quant_i8(wsvd_ctx *ctx, const void *gate_up, int64_t rows, int64_t F, int8_t *codes, void *scale_f16,
                                 void *hip_stream);

/*
 * Per-token symmetric int8 quantisation of activation rows (Section 4.2), same rounding rules as the
 * I8 latent quantiser with one scale per row of `cols` channels.
 *   x [rows, cols] of x_dtype (F32 or BF16) -> codes int8 [rows, cols], scale fp16 [rows].
 */
wsvd_status wsvd_quantize_act_i8(wsvd_ctx *ctx, const void *x, int32_t x_dtype, int64_t rows, int64_t cols,
                                 int8_t *codes, void *scale_f16, void *hip_stream);

/*
 * int4-weight x int8-activation linear layer (Section 4.2: per-channel symmetric weights, per-token
 * symmetric activations): out[m,n] = (sum_k x[m,k] * w[n,k]) * x_scale[m] * w_scale[n], the sum
 * exact in int32.
 *   x int8 [M,K]; x_scale fp16 [M]; w_i4 [N, K/2] two's-complement nibbles, element 2i in the low
 *   nibble of byte i; w_scale fp16 [N]; out [M,N] F32.  K multiple of 64 and <= 65536, N multiple of 32,
 *   M <= 64.  All DEVICE pointers; x, w_i4 and out 16-byte aligned.
 */
wsvd_status wsvd_linear_w4a8(wsvd_ctx *ctx, const int8_t *x, const void *x_scale, const void *w_i4,
                             const void *w_scale_f16, int64_t M, int64_t K, int64_t N, void *out,
                             int32_t out_dtype, void *hip_stream);

/*
 * The same layer with its output columns delivered as two row-major matrices: columns [0, n_first) to
 * out_first [M, n_first], columns [n_first, N) to out_rest [M, N - n_first].  One launch then serves the query
 * projection and the latent down-projection of the quantised block (weight rows W_Q, then A_K, then A_V; Section
 * 4.2 runs all of them in the same precision on the same activations): out_first is the query wsvd_decode_attn
 * takes, out_rest the latents wsvd_latent_store takes.  n_first a multiple of 32, 0 < n_first <= N.
 */
wsvd_status wsvd_linear_w4a8_split(wsvd_ctx *ctx, const int8_t *x, const void *x_scale, const void *w_i4,
                                   const void *w_scale_f16, int64_t M, int64_t K, int64_t N, int64_t n_first,
                                   void *out_first, void *out_rest, int32_t out_dtype, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* WSVD_H */
