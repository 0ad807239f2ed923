// Host-side launchers of the kernel translation units (internal; not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/wsvd.h"

// Per-context tuning and test settings (wsvd_ctx_set_option); defaults = automatic.
struct wsvd_options {
  int wg_per_cu = 4;        // scales the number of wavefronts the attention grid aims for (4 = one resident round)
  int min_chunk = 0;        // smallest context chunk per attention workgroup (rows); 0 = automatic (256, and no split at all where none pays)
  int max_threads = 0;      // cap on the matrix-core attention kernels' workgroup size (0 = their launch bound)
  int append_mode = 0;      // n > 0: the append kernel with n equal d_model slices merged by the last arriver
  int append_helpers = -1;  // helpers per unit of the default append kernel (-1 = automatic, 0 or 2)
  int fused_step = 0;       // wsvd_decode_step: 0 two launches, 1 the single-launch kernel where one exists, 2 that or UNSUPPORTED
  int linear_direct = 0;    // W4A8 linear layers read operands straight from memory (no LDS staging)
  int static_limit_kib = 0; // wsvd_decode_attn_static: pretend the static array is this small (tests of the rejection; 0 = its size)
  int prefill_tiled = 0;    // the tiled prefill kernels also for small calls
  int project_shape = 0;    // kernel of the tiled prefill projection (0 = automatic)
  int step_deferred = 1;    // wsvd_decode_step: projection launch + attention launch that finishes the row: 1 where supported, 2 that or UNSUPPORTED
  int timeline_kernel = 0;  // profiling build, wsvd_decode_step: whose stamps are recorded: 0 the attention launch's, 1 the projection launch's
  int step_slices = 0;      // d_model slices of that projection launch (0 = automatic)
};

struct wsvd_ctx {
  wsvd_options opt;
  int device;
  int n_cu;
  int* err_word;     // device, 4 bytes
  void* ws;          // caller-owned workspace
  size_t ws_bytes;
  int epoch;         // number of fused decode steps launched so far (value the append workgroups publish)
  void* static_scratch;   // this device's copy of the library's static scratch array (wsvd_decode_attn_static)
  long long* timeline;    // profiling build: caller's stamp buffer (wsvd_timeline_set_buffer), else null
  size_t timeline_bytes;
};

struct AttnParams;
struct AppendParams;

hipError_t wsvd_launch_quantize_rows(int latent_dtype, int rank, const float* c, int64_t n_rows, void* codes, void* meta,
                                     hipStream_t s);
hipError_t wsvd_launch_cache_copy(bool to_device, const wsvd_layer_desc& d, int plane, void* logical_codes,
                                  void* logical_meta, int t0, int n_rows, void* dev_codes, void* dev_meta, hipStream_t s);
hipError_t wsvd_launch_stream_read(const void* ptr, size_t bytes, int workgroups, int* sink, hipStream_t s);
hipError_t wsvd_launch_quantize_act_i8(const void* x, int x_dtype, int64_t rows, int64_t cols, int8_t* codes,
                                       void* scale_f16, hipStream_t s);
// d.batch = rows of x.  one_seq < 0: row b is the next token of sequence b; one_seq >= 0: all rows are consecutive
// tokens of that sequence.
hipError_t wsvd_launch_append(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale,
                              const void* A_K, const void* A_V, const wsvd_cache& cache, hipStream_t s, int one_seq = -1,
                              const wsvd_paged_cache* paged = nullptr);
hipError_t wsvd_launch_latent_store(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const float* cK, const float* cV,
                                    int64_t ld, const wsvd_cache& cache, hipStream_t s);
hipError_t wsvd_launch_pack_factor_a(const wsvd_layer_desc& d, const void* src, void* dst, hipStream_t s);
hipError_t wsvd_launch_attn(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* q, const void* q_scale,
                            const void* B_K, const void* B_V, const wsvd_cache& cache, int max_seq_len, void* out,
                            hipStream_t s);
// output columns [0, n_first) go to out (row-major [M, n_first]), the rest to out2 ([M, N - n_first])
void wsvd_attn_plan(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* q, const void* q_scale, const void* B_K,
                    const void* B_V, const wsvd_cache& cache, int max_seq_len, void* out, AttnParams& p, dim3& grid, int& threads,
                    int force_threads);
void wsvd_append_params(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale, const void* A_K,
                        const void* A_V, const wsvd_cache& cache, AppendParams& p);
int wsvd_append_mfma_waves(const wsvd_ctx* ctx, const wsvd_layer_desc& d);
bool wsvd_append_uses_mfma(const wsvd_layer_desc& d);
hipError_t wsvd_launch_attn_rope(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* q, const void* q_scale,
                                 const void* B_K, const void* B_V, const wsvd_cache& cache, int max_seq_len, double rope_base,
                                 void* out, hipStream_t s);
hipError_t wsvd_launch_attn_latent(const AttnParams& p, int latent_dtype, int rank, dim3 grid, int threads, hipStream_t s);
hipError_t wsvd_launch_attn_multi(const AttnParams& p, int rank, dim3 grid, int threads, hipStream_t s);
// tiled causal attention of nq query tokens per sequence (I8 latents, BF16 factors and queries); any nq
hipError_t wsvd_launch_prefill_attn(const wsvd_layer_desc& d, const void* q, int nq, int n_after, const void* B_K, const void* B_V,
                                    const wsvd_cache& cache, void* out, hipStream_t s,
                                    const wsvd_paged_cache* paged = nullptr);
// projection + quantise + store of n_tok consecutive tokens of sequence seq, or of every sequence when seq < 0 (x then
// holds [batch, n_tok, d_model]); I8 latents, BF16 x and factors; any n_tok
hipError_t wsvd_launch_prefill_project(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, int n_tok, int seq,
                                       const void* A_K, const void* A_V, const wsvd_cache& cache, hipStream_t s,
                                       const wsvd_paged_cache* paged = nullptr);
// decode attention over one shared rank-R latent (32 heads, rank 256 / 512 / 1024, int8 codes, bf16 q and factors):
// three launches (query absorption, attention with split partials, merge + output projection)
size_t wsvd_shared_ws_bytes(int batch, int rank, int t_cap);
hipError_t wsvd_launch_attn_shared(int batch, int d_head, int rank, int t_cap, float sm_scale, const void* q, const void* B_K,
                                   const void* B_V, const void* k_codes, const void* v_codes, const void* k_scale,
                                   const void* v_scale, const int* seq_lens, void* workspace, void* out, hipStream_t s);
hipError_t wsvd_launch_rmsnorm_quant(const float* x, const float* y_add, const float* gain, float eps, int64_t rows,
                                     int64_t cols, float* x_out, int8_t* codes, void* scale_f16, hipStream_t s);
hipError_t wsvd_launch_swiglu_quant(const float* gate_up, int64_t rows, int64_t F, int8_t* codes, void* scale_f16, hipStream_t s);
hipError_t wsvd_launch_fold_qk(const void* BQ, const void* BK, int factor_dtype, int Hq, int Hkv, int rq, int r, int d, float* out,
                               hipStream_t s);
hipError_t wsvd_launch_fold_vo(const void* BV, int factor_dtype, const float* WO, int E, int Hq, int Hkv, int r, int d, float* out,
                               hipStream_t s);
// hipErrorNotSupported when there is no fused kernel for the combination
hipError_t wsvd_launch_decode_step(wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* x_scale, const void* A_K,
                                   const void* A_V, const void* q, const void* q_scale, const void* B_K, const void* B_V,
                                   const wsvd_cache& cache, int max_seq_len, void* out, hipStream_t s);
hipError_t wsvd_launch_linear_w4a8(const int8_t* x, const void* x_scale, const void* w_i4, const void* w_scale, int64_t M,
                                   int64_t K, int64_t N, float* out, int64_t n_first, float* out2, bool direct, hipStream_t s);


// workspace sizing shared by the API and the launchers
size_t wsvd_attn_partial_floats(const wsvd_layer_desc& d);
hipError_t wsvd_launch_attn_gqa_store(const struct AttnParams& p, int rank, dim3 grid, int threads, hipStream_t s);
hipError_t wsvd_launch_attn_newrow(const struct AttnParams& p, int rank, dim3 grid, int threads, hipStream_t s);
bool wsvd_step_deferred_ok(const wsvd_layer_desc& d);
bool wsvd_step_partials(const wsvd_ctx* ctx, const wsvd_layer_desc& d, float** parts, int** pending, int* n_parts);
hipError_t wsvd_launch_append_project(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* x, const void* A_K,
                                      const void* A_V, const wsvd_cache& cache, float** parts, int** pending, int* n_parts,
                                      hipStream_t s);
size_t wsvd_attn_split_bytes(const wsvd_ctx* ctx, const wsvd_layer_desc& d, int max_seq_len);
size_t wsvd_append_partial_floats(const wsvd_layer_desc& d);
int wsvd_append_esplits(const wsvd_ctx* ctx, const wsvd_layer_desc& d);
