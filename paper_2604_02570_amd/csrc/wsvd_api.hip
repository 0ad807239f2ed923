// C ABI of the library: argument validation on the host, then kernel launches on the caller's stream.
#include <cstring>
#include <mutex>
#include <new>

#include "wsvd_attn_common.h"
#include "wsvd_internal.h"

hipError_t wsvd_launch_attn_generic(const AttnParams& p, int latent_dtype, int rank, dim3 grid, hipStream_t s);
hipError_t wsvd_launch_attn_mfma(const AttnParams& p, int latent_dtype, int rank, dim3 grid, int threads, hipStream_t s);
int wsvd_attn_mfma_max_threads(int latent_dtype, int rank, int G);
int wsvd_attn_mfma_waves_per_cu(int latent_dtype, int rank, int G);


// ---------------------------------------------------------------- static scratch of wsvd_decode_attn_static
// Device memory that belongs to the library image: one copy per GPU the library runs on, held until the process ends.
// Laid out like a caller's workspace (tickets first, then the split partials).  Host code never uses the array's name
// as an address: g_scratch_dev[device] holds what hipGetSymbolAddress returned with that device current.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_dev[kMaxDevices];          // per device; written once under g_scratch_mutex
static std::mutex g_scratch_mutex;

__global__ void k_fill_zero_i32(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Address of this device's copy of the array (the device must be current); looked up and its ticket region cleared
// the first time a context is created on the device.
static hipError_t static_scratch_for_device(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_dev[device]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    e = hipMemset(ptr, 0, (size_t)kWsCounterInts * 4);
    if (e != hipSuccess) return e;
    e = hipDeviceSynchronize();
    if (e != hipSuccess) return e;
    g_scratch_dev[device] = ptr;
  }
  *out = g_scratch_dev[device];
  return hipSuccess;
}

namespace {

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
inline bool is_pow2_rank(int r) { return r == 16 || r == 32 || r == 64; }
// ranks 96 and 128: int8 latents, one query head per kv head (other ranks are zero-padded up to a supported one)
inline bool is_wide_rank(int r) { return r == 96 || r == 128; }


wsvd_status check_desc(const wsvd_layer_desc* d) {
  if (!d) return WSVD_E_NULL;
  if (d->batch <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->d_model <= 0 || d->d_model % 64 != 0) return WSVD_E_SHAPE;
  if (d->d_head != 64 && d->d_head != 128) return WSVD_E_SHAPE;
  if (!is_pow2_rank(d->rank) && !is_wide_rank(d->rank)) return WSVD_E_SHAPE;
  if (is_wide_rank(d->rank) && (d->latent_dtype != WSVD_I8 || d->n_q_heads != d->n_kv_heads || d->d_head != 128)) return WSVD_E_UNSUPPORTED;
  if (d->n_q_heads % d->n_kv_heads != 0) return WSVD_E_SHAPE;
  const int G = d->n_q_heads / d->n_kv_heads;
  if (G < 1 || G > 8) return WSVD_E_SHAPE;
  if (d->t_cap <= 0 || d->t_cap % 64 != 0) return WSVD_E_SHAPE;
  if ((int64_t)d->batch * d->n_kv_heads > kWsCounterInts / 4) return WSVD_E_SHAPE;
  if (d->out_dtype != WSVD_F32 && d->out_dtype != WSVD_BF16) return WSVD_E_DTYPE;
  switch (d->latent_dtype) {
    case WSVD_F32:
      if (d->factor_dtype != WSVD_F32 || d->x_dtype != WSVD_F32 || d->q_dtype != WSVD_F32) return WSVD_E_DTYPE;
      break;
    case WSVD_BF16:
      if (d->factor_dtype != WSVD_BF16 || d->x_dtype != WSVD_BF16 || d->q_dtype != WSVD_BF16) return WSVD_E_DTYPE;
      break;
    case WSVD_I8:
    case WSVD_I4:
      if (d->factor_dtype != WSVD_BF16) return WSVD_E_DTYPE;
      if (d->x_dtype != WSVD_BF16 && d->x_dtype != WSVD_F32 && d->x_dtype != WSVD_I8) return WSVD_E_DTYPE;
      if (d->q_dtype != WSVD_I8 && d->q_dtype != WSVD_F32 && d->q_dtype != WSVD_BF16) return WSVD_E_DTYPE;
      if (d->latent_dtype == WSVD_I8 && d->rank != 32 && d->rank != 64 && !is_wide_rank(d->rank)) return WSVD_E_UNSUPPORTED;
      if (d->latent_dtype == WSVD_I4 && d->rank != 32) return WSVD_E_UNSUPPORTED;
      break;
    default:
      return WSVD_E_DTYPE;
  }
  return WSVD_OK;
}

int row_bytes_host(const wsvd_layer_desc& d) {
  switch (d.latent_dtype) {
    case WSVD_F32: return d.rank * 4;
    case WSVD_BF16: return d.rank * 2;
    case WSVD_I8: return d.rank;
    default: return d.rank / 2;
  }
}
int meta_bytes_host(const wsvd_layer_desc& d) { return d.latent_dtype == WSVD_I8 ? 2 : d.latent_dtype == WSVD_I4 ? 4 : 0; }

wsvd_status check_cache(const wsvd_layer_desc& d, const wsvd_cache* c) {
  if (!c || !c->k_codes || !c->v_codes || !c->seq_lens) return WSVD_E_NULL;
  const bool quant = d.latent_dtype == WSVD_I8 || d.latent_dtype == WSVD_I4;
  if (quant && (!c->k_meta || !c->v_meta)) return WSVD_E_NULL;
  if (!aligned16(c->k_codes) || !aligned16(c->v_codes) || !aligned16(c->k_meta) || !aligned16(c->v_meta) ||
      ((uintptr_t)c->seq_lens & 3u))
    return WSVD_E_ALIGN;
  return WSVD_OK;
}

}  // namespace

// size of the attention's split area in 4-byte units: one 8-byte word per (sequence, head, chunk, m | l | u_j), for
// the largest number of chunks a launch policy can choose (chunks are at least 256 rows)
size_t wsvd_attn_partial_floats(const wsvd_layer_desc& d) {
  const size_t max_chunks = (size_t)(d.t_cap + 255) / 256;
  // (the kernels for 5..8 query heads per kv head hand over up-projected vectors of d_head elements instead of rank)
  const size_t vec = (size_t)(d.rank > d.d_head ? d.rank : d.d_head) + 2;
  return 2 * (size_t)d.batch * d.n_q_heads * max_chunks * vec;
}

extern "C" {

const char* wsvd_status_str(wsvd_status s) {
  switch (s) {
    case WSVD_OK: return "ok";
    case WSVD_E_NULL: return "null pointer";
    case WSVD_E_SHAPE: return "unsupported or inconsistent shape";
    case WSVD_E_DTYPE: return "unsupported dtype combination";
    case WSVD_E_ALIGN: return "pointer not 16-byte aligned";
    case WSVD_E_CAPACITY: return "sequence at cache capacity";
    case WSVD_E_UNSUPPORTED: return "not implemented in this build";
    case WSVD_E_HIP: return "HIP runtime error";
    case WSVD_E_WORKSPACE: return "workspace missing or too small";
  }
  return "unknown status";
}

wsvd_status wsvd_create(wsvd_ctx** out, int device_ordinal) {
  if (!out) return WSVD_E_NULL;
  *out = nullptr;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess) return WSVD_E_HIP;
  if (device_ordinal < 0 || device_ordinal >= n_dev) return WSVD_E_SHAPE;
  if (hipSetDevice(device_ordinal) != hipSuccess) return WSVD_E_HIP;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device_ordinal) != hipSuccess) return WSVD_E_HIP;
  wsvd_ctx* c = new (std::nothrow) wsvd_ctx();
  if (!c) return WSVD_E_HIP;
  c->device = device_ordinal;
  c->n_cu = prop.multiProcessorCount;
  c->ws = nullptr;
  c->ws_bytes = 0;
  c->epoch = 0;
  c->timeline = nullptr;
  c->timeline_bytes = 0;
  if (hipMalloc((void**)&c->err_word, 4) != hipSuccess) { delete c; return WSVD_E_HIP; }
  if (hipMemset(c->err_word, 0, 4) != hipSuccess) { (void)hipFree(c->err_word); delete c; return WSVD_E_HIP; }
  if (static_scratch_for_device(device_ordinal, &c->static_scratch) != hipSuccess) { (void)hipFree(c->err_word); delete c; return WSVD_E_HIP; }
  *out = c;
  return WSVD_OK;
}

wsvd_status wsvd_destroy(wsvd_ctx* ctx) {
  if (!ctx) return WSVD_E_NULL;
  hipError_t e = hipFree(ctx->err_word);
  delete ctx;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_cache_bytes(const wsvd_layer_desc* desc, size_t* codes_bytes, size_t* meta_bytes) {
  if (!codes_bytes || !meta_bytes) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  const size_t rows = (size_t)desc->batch * desc->n_kv_heads * desc->t_cap;
  *codes_bytes = rows * row_bytes_host(*desc);
  *meta_bytes = rows * meta_bytes_host(*desc);
  return WSVD_OK;
}

wsvd_status wsvd_workspace_bytes(const wsvd_layer_desc* desc, size_t* bytes) {
  if (!bytes) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  const size_t a = wsvd_attn_partial_floats(*desc), b = wsvd_append_partial_floats(*desc);
  // counters, the attention's split words, the append's pushed words, the sliced append's partial sums (16-byte aligned)
  *bytes = (size_t)kWsCounterInts * 4 + ((a + 3) / 4 * 4 + b) * 4;
  return WSVD_OK;
}

wsvd_status wsvd_set_workspace(wsvd_ctx* ctx, void* dev_ptr, size_t bytes) {
  if (!ctx || !dev_ptr) return WSVD_E_NULL;
  if (!aligned16(dev_ptr)) return WSVD_E_ALIGN;
  if (bytes < (size_t)kWsCounterInts * 4) return WSVD_E_WORKSPACE;
  if (hipSetDevice(ctx->device) != hipSuccess) return WSVD_E_HIP;
  // tickets, flags and the append's pushed words all start at zero and are left at zero by every launch
  if (hipMemset(dev_ptr, 0, bytes) != hipSuccess) return WSVD_E_HIP;
  if (hipDeviceSynchronize() != hipSuccess) return WSVD_E_HIP;
  ctx->ws = dev_ptr;
  ctx->ws_bytes = bytes;
  return WSVD_OK;
}

// Settings of one context: work decomposition (tuning) and the choice between alternative kernels (tests).
wsvd_status wsvd_ctx_set_option(wsvd_ctx* ctx, const char* name, int value) {
  if (!ctx || !name) return WSVD_E_NULL;
  wsvd_options& o = ctx->opt;
  if (!strcmp(name, "wg_per_cu") && value >= 1 && value <= 64) { o.wg_per_cu = value; return WSVD_OK; }
  if (!strcmp(name, "min_chunk") && value >= 0 && value % 64 == 0) { o.min_chunk = value; return WSVD_OK; }
  if (!strcmp(name, "max_threads") && (value == 0 || (value >= 256 && value <= 1024 && value % 256 == 0))) { o.max_threads = value; return WSVD_OK; }
  if (!strcmp(name, "append_mode") && value >= 0 && value <= 64) { o.append_mode = value; return WSVD_OK; }
  if (!strcmp(name, "append_helpers") && (value == -1 || value == 0 || value == 2)) { o.append_helpers = value; return WSVD_OK; }
  if (!strcmp(name, "fused_step") && value >= 0 && value <= 2) { o.fused_step = value; return WSVD_OK; }
  if (!strcmp(name, "static_limit_kib") && value >= 0 && value <= (int)(kStaticScratchBytes >> 10)) { o.static_limit_kib = value; return WSVD_OK; }
  if (!strcmp(name, "linear_direct") && value >= 0 && value <= 1) { o.linear_direct = value; return WSVD_OK; }
  if (!strcmp(name, "prefill_tiled") && value >= 0 && value <= 1) { o.prefill_tiled = value; return WSVD_OK; }
  if (!strcmp(name, "step_deferred") && value >= 0 && value <= 2) { o.step_deferred = value; return WSVD_OK; }
  if (!strcmp(name, "timeline_kernel") && value >= 0 && value <= 1) { o.timeline_kernel = value; return WSVD_OK; }
  if (!strcmp(name, "step_slices") && value >= 0 && value <= 4) { o.step_slices = value; return WSVD_OK; }
  if (!strcmp(name, "project_shape") && (value == 0 || value == 1 || value == 2 || value == 21 || value == 24 || value == 42 || value == 44)) { o.project_shape = value; return WSVD_OK; }
  return WSVD_E_SHAPE;
}

wsvd_status wsvd_latent_append(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* x, const void* x_scale,
                               const void* A_K, const void* A_V, wsvd_cache* cache, void* hip_stream) {
  if (!ctx || !x || !A_K || !A_V) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->x_dtype == WSVD_I8 && !x_scale) return WSVD_E_NULL;
  if (!aligned16(x) || !aligned16(A_K) || !aligned16(A_V)) return WSVD_E_ALIGN;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  hipError_t e = wsvd_launch_append(ctx, *desc, x, x_scale, A_K, A_V, *cache, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_prefill_append(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* x, const void* x_scale, int32_t n_tokens,
                                int32_t seq_index, const void* A_K, const void* A_V, wsvd_cache* cache, void* hip_stream) {
  if (!ctx || !x || !A_K || !A_V) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->x_dtype == WSVD_I8 && !x_scale) return WSVD_E_NULL;
  if (!aligned16(x) || !aligned16(A_K) || !aligned16(A_V)) return WSVD_E_ALIGN;
  if (n_tokens < 1 || seq_index < -1 || seq_index >= desc->batch) return WSVD_E_SHAPE;
  const bool i4 = desc->latent_dtype == WSVD_I4;
  if (n_tokens > 64 || seq_index < 0 || ctx->opt.prefill_tiled || desc->rank > 64 || i4) {
    // a prompt-sized block, or all sequences at once, or int4 latents (whose value bytes pair two rows: only the tiled
    // kernel writes both rows of a byte from one place): the tiled projection (one launch for all its tokens)
    const bool fits = (desc->latent_dtype == WSVD_I8 || i4) && desc->factor_dtype == WSVD_BF16 && desc->x_dtype == WSVD_BF16;
    if (!fits && i4) return WSVD_E_UNSUPPORTED;
    if (!fits && desc->rank > 64) return WSVD_E_UNSUPPORTED;
    if (!fits && (n_tokens > 64 || seq_index < 0)) return WSVD_E_SHAPE;
    if (fits) {
      hipError_t e = wsvd_launch_prefill_project(ctx, *desc, x, n_tokens, seq_index, A_K, A_V, *cache, (hipStream_t)hip_stream);
      if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
      return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
    }
  }
  wsvd_layer_desc d = *desc;
  d.batch = n_tokens;                       // rows of x in this launch
  size_t need;
  wsvd_workspace_bytes(&d, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  hipError_t e = wsvd_launch_append(ctx, d, x, x_scale, A_K, A_V, *cache, (hipStream_t)hip_stream, seq_index);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_prefill_attn(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* q, int32_t n_q, int32_t n_after,
                              const void* B_K, const void* B_V, const wsvd_cache* cache, int32_t max_seq_len, void* out,
                              void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (desc->out_dtype != WSVD_F32) return WSVD_E_UNSUPPORTED;       // the prompt kernels write fp32
  const int Gr = desc->n_q_heads / desc->n_kv_heads;
  if (n_q < 1 || n_after < 0 || max_seq_len < 0) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  if (desc->q_dtype == WSVD_I8) return WSVD_E_DTYPE;          // one scale per sequence cannot serve several tokens
  if (desc->latent_dtype != WSVD_I8 || desc->factor_dtype != WSVD_BF16 || desc->rank > 64) return WSVD_E_UNSUPPORTED;
  if ((int64_t)n_q * Gr > 8 || (ctx->opt.prefill_tiled && desc->q_dtype == WSVD_BF16)) {
    // more query rows than the decode kernel has slots: the tiled kernel (one wavefront per 32 query rows)
    if (desc->q_dtype != WSVD_BF16) return WSVD_E_UNSUPPORTED;
    hipError_t e = wsvd_launch_prefill_attn(*desc, q, n_q, n_after, B_K, B_V, *cache, out, (hipStream_t)hip_stream);
    if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
    return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
  }
  wsvd_layer_desc d = *desc;
  d.n_q_heads = desc->n_kv_heads * n_q * Gr;                  // query slots take the place of query heads
  size_t need;
  wsvd_workspace_bytes(&d, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  AttnParams p;
  dim3 grid;
  int threads;
  wsvd_attn_plan(ctx, d, q, nullptr, B_K, B_V, *cache, max_seq_len, out, p, grid, threads, 0);
  if (threads > 512) wsvd_attn_plan(ctx, d, q, nullptr, B_K, B_V, *cache, max_seq_len, out, p, grid, threads, 512);
  p.nq = n_q; p.Gr = Gr; p.n_after = n_after;
  hipError_t e = wsvd_launch_attn_multi(p, d.rank, grid, threads, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

namespace {
wsvd_status check_shared(int32_t batch, int32_t n_heads, int32_t d_head, int32_t rank, int32_t t_cap) {
  if (batch < 1 || t_cap < 128 || t_cap % 128 != 0) return WSVD_E_SHAPE;
  if (d_head != 64 && d_head != 128) return WSVD_E_SHAPE;
  if (n_heads != 32) return WSVD_E_UNSUPPORTED;                    // the heads are the 32 columns of the matrix products
  const bool wide = rank > 1024 && rank <= 4096 && rank % 128 == 0;    // walked in slabs of 1024: up to 16384 cached tokens
  if (rank != 256 && rank != 512 && rank != 1024 && !wide) return WSVD_E_UNSUPPORTED;
  if (wide && t_cap > 16384) return WSVD_E_UNSUPPORTED;
  return WSVD_OK;
}
}  // namespace

wsvd_status wsvd_shared_workspace_bytes(int32_t batch, int32_t n_heads, int32_t d_head, int32_t rank, int32_t t_cap, size_t* bytes) {
  if (!bytes) return WSVD_E_NULL;
  wsvd_status st = check_shared(batch, n_heads, d_head, rank, t_cap);
  if (st != WSVD_OK) return st;
  *bytes = wsvd_shared_ws_bytes(batch, rank, t_cap);
  return WSVD_OK;
}

wsvd_status wsvd_decode_attn_shared(wsvd_ctx* ctx, int32_t batch, int32_t n_heads, int32_t d_head, int32_t rank, int32_t t_cap,
                                    float sm_scale, const void* q, const void* B_K, const void* B_V, const void* k_codes,
                                    const void* v_codes, const void* k_scale, const void* v_scale, const int32_t* seq_lens,
                                    void* workspace, size_t workspace_bytes, void* out, void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !k_codes || !v_codes || !k_scale || !v_scale || !seq_lens || !workspace || !out) return WSVD_E_NULL;
  wsvd_status st = check_shared(batch, n_heads, d_head, rank, t_cap);
  if (st != WSVD_OK) return st;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(k_codes) || !aligned16(v_codes) || !aligned16(k_scale) ||
      !aligned16(v_scale) || !aligned16(workspace) || !aligned16(out) || ((uintptr_t)seq_lens & 3u))
    return WSVD_E_ALIGN;
  if (workspace_bytes < wsvd_shared_ws_bytes(batch, rank, t_cap)) return WSVD_E_WORKSPACE;
  const float sm = sm_scale > 0.f ? sm_scale : 1.0f / sqrtf((float)d_head);
  hipError_t e = wsvd_launch_attn_shared(batch, d_head, rank, t_cap, sm, q, B_K, B_V, k_codes, v_codes, k_scale, v_scale, seq_lens,
                                         workspace, out, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_decode_attn_rope(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* q, const void* q_scale,
                                  const void* B_K, const void* B_V, const wsvd_cache* cache, int32_t max_seq_len,
                                  float rope_base, void* out, void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->q_dtype == WSVD_I8 && !q_scale) return WSVD_E_NULL;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (max_seq_len < 0 || !(rope_base > 1.0f)) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  if (desc->rank > 64) return WSVD_E_UNSUPPORTED;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  hipError_t e = wsvd_launch_attn_rope(ctx, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, (double)rope_base, out,
                                       (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_latent_store(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const float* c_K, const float* c_V, int64_t ld,
                              wsvd_cache* cache, void* hip_stream) {
  if (!ctx || !c_K || !c_V) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (ld < (int64_t)desc->n_kv_heads * desc->rank) return WSVD_E_SHAPE;
  if (desc->rank > 64) return WSVD_E_UNSUPPORTED;
  if (((uintptr_t)c_K & 3u) || ((uintptr_t)c_V & 3u)) return WSVD_E_ALIGN;
  hipError_t e = wsvd_launch_latent_store(ctx, *desc, c_K, c_V, ld, *cache, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_decode_attn(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* q, const void* q_scale,
                             const void* B_K, const void* B_V, const wsvd_cache* cache, int32_t max_seq_len, void* out,
                             void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->q_dtype == WSVD_I8 && !q_scale) return WSVD_E_NULL;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (max_seq_len < 0) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  hipError_t e = wsvd_launch_attn(ctx, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, out, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_decode_attn_store(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const float* c_K, const float* c_V, int64_t ld,
                                   const void* q, const void* q_scale, const void* B_K, const void* B_V, wsvd_cache* cache,
                                   int32_t max_seq_len, void* out, void* hip_stream) {
  if (!ctx || !c_K || !c_V || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->q_dtype == WSVD_I8 && !q_scale) return WSVD_E_NULL;
  if (ld < (int64_t)desc->n_kv_heads * desc->rank) return WSVD_E_SHAPE;
  if (desc->rank > 64) return WSVD_E_UNSUPPORTED;
  if (((uintptr_t)c_K & 3u) || ((uintptr_t)c_V & 3u)) return WSVD_E_ALIGN;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (max_seq_len < 1) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  const int G = desc->n_q_heads / desc->n_kv_heads;
  if (desc->latent_dtype == WSVD_I8 && G > 4 && desc->batch <= 8192) {
    AttnParams p;
    dim3 grid;
    int threads;
    wsvd_attn_plan(ctx, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, out, p, grid, threads, 0);
    p.new_k = c_K; p.new_v = c_V; p.new_ld = (long)ld;
    p.done = (int*)ctx->ws;                   // one counter per sequence, zero between launches
    p.seq_lens_rw = cache->seq_lens;
    hipError_t e = wsvd_launch_attn_gqa_store(p, desc->rank, grid, threads, s);
    if (e != hipErrorNotSupported) return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
  }
  // no single-launch kernel for this combination: the two calls back to back on the stream
  hipError_t e = wsvd_launch_latent_store(ctx, *desc, c_K, c_V, ld, *cache, s);
  if (e == hipSuccess) e = wsvd_launch_attn(ctx, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, out, s);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

namespace {
wsvd_status check_paged(const wsvd_layer_desc& d, const wsvd_paged_cache* c) {
  if (!c || !c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta || !c->seq_lens || !c->block_table) return WSVD_E_NULL;
  if (d.latent_dtype != WSVD_I8 && d.latent_dtype != WSVD_I4) return WSVD_E_UNSUPPORTED;
  if (d.rank > 64) return WSVD_E_UNSUPPORTED;
  if (c->page_rows < 64 || c->page_rows % 64 != 0 || c->max_pages < 1 || c->n_pages < 1) return WSVD_E_SHAPE;
  if ((int64_t)c->max_pages * c->page_rows != d.t_cap) return WSVD_E_SHAPE;
  if (!aligned16(c->k_codes) || !aligned16(c->v_codes) || !aligned16(c->k_meta) || !aligned16(c->v_meta) ||
      ((uintptr_t)c->seq_lens & 3u) || ((uintptr_t)c->block_table & 3u))
    return WSVD_E_ALIGN;
  return WSVD_OK;
}
}  // namespace

wsvd_status wsvd_paged_cache_bytes(const wsvd_layer_desc* desc, int32_t page_rows, int32_t n_pages, size_t* codes_bytes,
                                   size_t* meta_bytes) {
  if (!codes_bytes || !meta_bytes) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if (page_rows < 64 || page_rows % 64 != 0 || n_pages < 1) return WSVD_E_SHAPE;
  *codes_bytes = (size_t)n_pages * desc->n_kv_heads * page_rows * row_bytes_host(*desc);
  *meta_bytes = (size_t)n_pages * desc->n_kv_heads * page_rows * meta_bytes_host(*desc);
  return WSVD_OK;
}

wsvd_status wsvd_latent_append_paged(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* x, const void* x_scale,
                                     const void* A_K, const void* A_V, wsvd_paged_cache* cache, void* hip_stream) {
  if (!ctx || !x || !A_K || !A_V) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_paged(*desc, cache)) != WSVD_OK) return st;
  if (desc->x_dtype == WSVD_I8 && !x_scale) return WSVD_E_NULL;
  if (!aligned16(x) || !aligned16(A_K) || !aligned16(A_V)) return WSVD_E_ALIGN;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  wsvd_cache view = {cache->k_codes, cache->v_codes, cache->k_meta, cache->v_meta, cache->seq_lens};
  hipError_t e = wsvd_launch_append(ctx, *desc, x, x_scale, A_K, A_V, view, (hipStream_t)hip_stream, -1, cache);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_prefill_append_paged(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* x, int32_t n_tokens, int32_t seq_index,
                                      const void* A_K, const void* A_V, wsvd_paged_cache* cache, void* hip_stream) {
  if (!ctx || !x || !A_K || !A_V) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_paged(*desc, cache)) != WSVD_OK) return st;
  if (desc->x_dtype != WSVD_BF16 || desc->factor_dtype != WSVD_BF16) return WSVD_E_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(A_K) || !aligned16(A_V)) return WSVD_E_ALIGN;
  if (n_tokens < 1 || seq_index < -1 || seq_index >= desc->batch) return WSVD_E_SHAPE;
  wsvd_cache view = {cache->k_codes, cache->v_codes, cache->k_meta, cache->v_meta, cache->seq_lens};
  hipError_t e = wsvd_launch_prefill_project(ctx, *desc, x, n_tokens, seq_index, A_K, A_V, view, (hipStream_t)hip_stream, cache);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_prefill_attn_paged(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* q, int32_t n_q, int32_t n_after,
                                    const void* B_K, const void* B_V, const wsvd_paged_cache* cache, int32_t max_seq_len, void* out,
                                    void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_paged(*desc, cache)) != WSVD_OK) return st;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (desc->out_dtype != WSVD_F32) return WSVD_E_UNSUPPORTED;
  if (n_q < 1 || n_after < 0 || max_seq_len < 0) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  if (desc->latent_dtype != WSVD_I8 || desc->factor_dtype != WSVD_BF16 || desc->q_dtype != WSVD_BF16) return WSVD_E_UNSUPPORTED;
  wsvd_cache view = {cache->k_codes, cache->v_codes, cache->k_meta, cache->v_meta, cache->seq_lens};
  hipError_t e = wsvd_launch_prefill_attn(*desc, q, n_q, n_after, B_K, B_V, view, out, (hipStream_t)hip_stream, cache);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_decode_attn_paged(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* q, const void* q_scale,
                                   const void* B_K, const void* B_V, const wsvd_paged_cache* cache, int32_t max_seq_len,
                                   void* out, void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_paged(*desc, cache)) != WSVD_OK) return st;
  if (desc->q_dtype == WSVD_I8 && !q_scale) return WSVD_E_NULL;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (max_seq_len < 0) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  wsvd_cache view = {cache->k_codes, cache->v_codes, cache->k_meta, cache->v_meta, cache->seq_lens};
  AttnParams p;
  dim3 grid;
  int threads;
  wsvd_attn_plan(ctx, *desc, q, q_scale, B_K, B_V, view, max_seq_len, out, p, grid, threads, 0);
  p.block_table = cache->block_table; p.page_rows = cache->page_rows; p.max_pages = cache->max_pages; p.n_pages = cache->n_pages;
  hipError_t e = wsvd_launch_attn_mfma(p, desc->latent_dtype, desc->rank, grid, threads, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_decode_attn_static(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* q, const void* q_scale,
                                    const void* B_K, const void* B_V, const wsvd_cache* cache, int32_t max_seq_len, void* out,
                                    void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->q_dtype == WSVD_I8 && !q_scale) return WSVD_E_NULL;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (max_seq_len < 0) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  // counters + the split words of this launch must fit the static array
  const size_t need = (size_t)kWsCounterInts * 4 + wsvd_attn_split_bytes(ctx, *desc, max_seq_len);
  const size_t limit = ctx->opt.static_limit_kib ? (size_t)ctx->opt.static_limit_kib << 10 : kStaticScratchBytes;
  if (need > limit) return WSVD_E_WORKSPACE;
  if (!ctx->static_scratch) return WSVD_E_HIP;
  hipStream_t s = (hipStream_t)hip_stream;
  // the same launch as wsvd_decode_attn, with the array in the caller's workspace's place (a copy of the context on
  // the stack: the caller's own workspace setting is left alone)
  wsvd_ctx view = *ctx;
  view.ws = ctx->static_scratch;
  view.ws_bytes = kStaticScratchBytes;
  // The split words must start at zero.  Their consumer clears them at the end of every launch, but the array
  // outlives every call (also one that was cut short), so the part this launch uses is cleared on the stream first: a
  // fill kernel, not a memset node, so that the call can be captured into a graph.
  const size_t split_bytes = need - (size_t)kWsCounterInts * 4;
  if (split_bytes) {
    const int n_ints = (int)(split_bytes / 4);
    hipLaunchKernelGGL(k_fill_zero_i32, dim3((n_ints + 255) / 256), dim3(256), 0, s, (int*)((char*)view.ws + (size_t)kWsCounterInts * 4), n_ints);
    if (hipGetLastError() != hipSuccess) return WSVD_E_HIP;
  }
  hipError_t e = wsvd_launch_attn(&view, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, out, s);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

// the second launch of the deferred-row decode step
static hipError_t launch_step_attention(wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* q, const void* q_scale, const void* B_K,
                                        const void* B_V, const wsvd_cache& cache, int max_seq_len, void* out, float* parts,
                                        int* pending, int n_parts, hipStream_t s) {
  AttnParams p;
  dim3 grid;
  int threads;
  wsvd_attn_plan(ctx, d, q, q_scale, B_K, B_V, cache, max_seq_len, out, p, grid, threads, 0);
  const size_t plane = (size_t)d.batch * d.n_kv_heads * d.rank;
  p.new_k = parts; p.new_v = parts + plane; p.new_ld = (long)d.n_kv_heads * d.rank;
  p.n_parts = n_parts; p.part_stride = (long)(2 * plane); p.pending = pending;
  if (ctx->opt.timeline_kernel == 1) p.timeline = nullptr;
  return wsvd_launch_attn_newrow(p, d.rank, grid, threads, s);
}

wsvd_status wsvd_test_step_attention(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* q, const void* q_scale, const void* B_K,
                                     const void* B_V, wsvd_cache* cache, int32_t max_seq_len, void* out, void* hip_stream) {
  if (!ctx || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->q_dtype == WSVD_I8 && !q_scale) return WSVD_E_NULL;
  if (!aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out)) return WSVD_E_ALIGN;
  if (max_seq_len < 1) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  float* parts = nullptr;
  int* pending = nullptr;
  int n_parts = 0;
  if (!wsvd_step_deferred_ok(*desc) || !wsvd_step_partials(ctx, *desc, &parts, &pending, &n_parts)) return WSVD_E_UNSUPPORTED;
  hipError_t e = launch_step_attention(ctx, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, out, parts, pending, n_parts, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_decode_step(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* x, const void* x_scale, const void* A_K,
                             const void* A_V, const void* q, const void* q_scale, const void* B_K, const void* B_V,
                             wsvd_cache* cache, int32_t max_seq_len, void* out, void* hip_stream) {
  if (!ctx || !x || !A_K || !A_V || !q || !B_K || !B_V || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (desc->x_dtype == WSVD_I8 && !x_scale) return WSVD_E_NULL;
  if (desc->q_dtype == WSVD_I8 && !q_scale) return WSVD_E_NULL;
  if (!aligned16(x) || !aligned16(A_K) || !aligned16(A_V) || !aligned16(q) || !aligned16(B_K) || !aligned16(B_V) || !aligned16(out))
    return WSVD_E_ALIGN;
  if (max_seq_len < 1) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = ctx->opt.fused_step ? wsvd_launch_decode_step(ctx, *desc, x, x_scale, A_K, A_V, q, q_scale, B_K, B_V, *cache,
                                                            max_seq_len, out, s)
                                  : hipErrorNotSupported;
  if (e == hipErrorNotSupported && ctx->opt.fused_step == 2) return WSVD_E_UNSUPPORTED;
  if (e == hipErrorNotSupported && ctx->opt.step_deferred && ctx->opt.append_mode == 0 && wsvd_step_deferred_ok(*desc)) {
    // projection launch (partial sums, lengths advanced), then the attention launch that finishes the rows
    float* parts = nullptr;
    int* pending = nullptr;
    int n_parts = 0;
    e = wsvd_launch_append_project(ctx, *desc, x, A_K, A_V, *cache, &parts, &pending, &n_parts, s);
    if (e == hipSuccess) e = launch_step_attention(ctx, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, out, parts, pending, n_parts, s);
    if (e != hipErrorNotSupported) return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
  }
  if (e == hipErrorNotSupported && ctx->opt.step_deferred == 2) return WSVD_E_UNSUPPORTED;
  if (e == hipErrorNotSupported) {
    // no fused kernel for this combination: the two calls back to back on the stream
    e = wsvd_launch_append(ctx, *desc, x, x_scale, A_K, A_V, *cache, s);
    if (e == hipSuccess) e = wsvd_launch_attn(ctx, *desc, q, q_scale, B_K, B_V, *cache, max_seq_len, out, s);
    if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  }
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_factor_a_bytes(const wsvd_layer_desc* desc, size_t* bytes) {
  if (!bytes) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  *bytes = (size_t)desc->n_kv_heads * ((desc->rank + 31) / 32) * 32 * desc->d_model * (desc->factor_dtype == WSVD_F32 ? 4 : 2);
  return WSVD_OK;
}

wsvd_status wsvd_pack_factor_a(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* A_row_major, void* A_packed, void* hip_stream) {
  if (!ctx || !A_row_major || !A_packed) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if (!aligned16(A_row_major) || !aligned16(A_packed)) return WSVD_E_ALIGN;
  hipError_t e = wsvd_launch_pack_factor_a(*desc, A_row_major, A_packed, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_check(wsvd_ctx* ctx, void* hip_stream) {
  if (!ctx) return WSVD_E_NULL;
  hipStream_t s = (hipStream_t)hip_stream;
  int host = 0;
  if (hipMemcpyAsync(&host, ctx->err_word, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return WSVD_E_HIP;
  if (hipStreamSynchronize(s) != hipSuccess) return WSVD_E_HIP;
  if (host != 0) {
    if (hipMemsetAsync(ctx->err_word, 0, 4, s) != hipSuccess) return WSVD_E_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return WSVD_E_HIP;
  }
  return (wsvd_status)host;
}

wsvd_status wsvd_quantize_rows(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const float* c, int64_t n_rows, void* codes,
                               void* meta, void* hip_stream) {
  if (!ctx || !c || !codes || !meta) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if (desc->latent_dtype != WSVD_I8 && desc->latent_dtype != WSVD_I4) return WSVD_E_DTYPE;
  if (n_rows < 0) return WSVD_E_SHAPE;
  if (!aligned16(c) || !aligned16(codes) || !aligned16(meta)) return WSVD_E_ALIGN;
  hipError_t e = wsvd_launch_quantize_rows(desc->latent_dtype, desc->rank, c, n_rows, codes, meta, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

static wsvd_status cache_copy(bool to_device, wsvd_ctx* ctx, const wsvd_layer_desc* desc, int32_t plane, void* codes,
                              void* meta, int32_t t0, int32_t n_rows, const wsvd_cache* cache, void* hip_stream) {
  if (!ctx || !codes) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  const bool quant = desc->latent_dtype == WSVD_I8 || desc->latent_dtype == WSVD_I4;
  if (quant && !meta) return WSVD_E_NULL;
  if (plane != 0 && plane != 1) return WSVD_E_SHAPE;
  if (t0 < 0 || n_rows < 0 || (int64_t)t0 + n_rows > desc->t_cap) return WSVD_E_SHAPE;
  if (!aligned16(codes) || !aligned16(meta)) return WSVD_E_ALIGN;
  hipError_t e = wsvd_launch_cache_copy(to_device, *desc, plane, codes, meta, t0, n_rows,
                                        plane == 0 ? cache->k_codes : cache->v_codes,
                                        plane == 0 ? cache->k_meta : cache->v_meta, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_cache_import(wsvd_ctx* ctx, const wsvd_layer_desc* desc, int32_t which_plane, const void* codes,
                              const void* meta, int32_t t0, int32_t n_rows, wsvd_cache* cache, void* hip_stream) {
  return cache_copy(true, ctx, desc, which_plane, (void*)codes, (void*)meta, t0, n_rows, cache, hip_stream);
}

wsvd_status wsvd_cache_export(wsvd_ctx* ctx, const wsvd_layer_desc* desc, int32_t which_plane, const wsvd_cache* cache,
                              int32_t t0, int32_t n_rows, void* codes, void* meta, void* hip_stream) {
  return cache_copy(false, ctx, desc, which_plane, codes, meta, t0, n_rows, cache, hip_stream);
}

wsvd_status wsvd_decode_attn_latent(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* c_Q, int32_t rq, const void* qk_fold,
                                    const wsvd_cache* cache, int32_t max_seq_len, void* u_out, void* hip_stream) {
  if (!ctx || !c_Q || !qk_fold || !u_out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if ((st = check_cache(*desc, cache)) != WSVD_OK) return st;
  if (rq < 1 || rq > 64) return WSVD_E_SHAPE;
  if (!aligned16(c_Q) || !aligned16(qk_fold) || !aligned16(u_out)) return WSVD_E_ALIGN;
  if (max_seq_len < 0) return WSVD_E_SHAPE;
  if (max_seq_len > desc->t_cap) return WSVD_E_CAPACITY;
  const int G = desc->n_q_heads / desc->n_kv_heads;
  if (desc->latent_dtype != WSVD_I8 && desc->latent_dtype != WSVD_I4) return WSVD_E_UNSUPPORTED;
  if (G > 8 || desc->rank > 64) return WSVD_E_UNSUPPORTED;
  size_t need;
  wsvd_workspace_bytes(desc, &need);
  if (!ctx->ws || ctx->ws_bytes < need) return WSVD_E_WORKSPACE;
  wsvd_layer_desc d = *desc;
  d.q_dtype = WSVD_F32;                       // the Q latent arrives as the fp32 output of its projection
  AttnParams p;
  dim3 grid;
  int threads;
  wsvd_attn_plan(ctx, d, c_Q, nullptr, nullptr, nullptr, *cache, max_seq_len, u_out, p, grid, threads, G > 4 ? 512 : 0);
  p.qk_fold = (const float*)qk_fold;
  p.rq = rq;
  p.out_dim = d.rank;
  p.out_bf16 = 0;                              // the latent-space output is fp32 whatever the layer's output format
  hipError_t e = wsvd_launch_attn_latent(p, d.latent_dtype, d.rank, grid, threads, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_fold_qk(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* B_Q, int32_t rq, const void* B_K, void* out,
                         void* hip_stream) {
  if (!ctx || !B_Q || !B_K || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  if (rq < 1 || rq > 64) return WSVD_E_SHAPE;
  hipError_t e = wsvd_launch_fold_qk(B_Q, B_K, desc->factor_dtype, desc->n_q_heads, desc->n_kv_heads, rq, desc->rank, desc->d_head,
                                     (float*)out, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_fold_vo(wsvd_ctx* ctx, const wsvd_layer_desc* desc, const void* B_V, const void* W_O, void* out, void* hip_stream) {
  if (!ctx || !B_V || !W_O || !out) return WSVD_E_NULL;
  wsvd_status st = check_desc(desc);
  if (st != WSVD_OK) return st;
  hipError_t e = wsvd_launch_fold_vo(B_V, desc->factor_dtype, (const float*)W_O, desc->d_model, desc->n_q_heads, desc->n_kv_heads,
                                     desc->rank, desc->d_head, (float*)out, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_rmsnorm_quant_i8(wsvd_ctx* ctx, const void* x, const void* y_add, const void* gain, float eps, int64_t rows,
                                  int64_t cols, void* x_out, int8_t* codes, void* scale_f16, void* hip_stream) {
  if (!ctx || !x || !gain || !codes || !scale_f16) return WSVD_E_NULL;
  if (y_add && !x_out) return WSVD_E_NULL;
  if (rows < 0 || cols < 4 || cols % 4 != 0 || cols > 16384 || !(eps >= 0.f)) return WSVD_E_SHAPE;
  if (!aligned16(x) || !aligned16(gain) || !aligned16(codes) || (y_add && (!aligned16(y_add) || !aligned16(x_out)))) return WSVD_E_ALIGN;
  hipError_t e = wsvd_launch_rmsnorm_quant((const float*)x, (const float*)y_add, (const float*)gain, eps, rows, cols, (float*)x_out,
                                           codes, scale_f16, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_swiglu_quant_i8(wsvd_ctx* ctx, const void* gate_up, int64_t rows, int64_t F, int8_t* codes, void* scale_f16,
                                 void* hip_stream) {
  if (!ctx || !gate_up || !codes || !scale_f16) return WSVD_E_NULL;
  if (rows < 0 || F < 4 || F % 4 != 0 || F > 16384) return WSVD_E_SHAPE;
  if (!aligned16(gate_up) || !aligned16(codes)) return WSVD_E_ALIGN;
  hipError_t e = wsvd_launch_swiglu_quant((const float*)gate_up, rows, F, codes, scale_f16, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_timeline_set_buffer(wsvd_ctx* ctx, void* dev_ptr, size_t bytes) {
  if (!ctx) return WSVD_E_NULL;
#ifdef WSVD_TIMELINE
  if (dev_ptr && !aligned16(dev_ptr)) return WSVD_E_ALIGN;
  ctx->timeline = (long long*)dev_ptr;
  ctx->timeline_bytes = dev_ptr ? bytes : 0;
  return WSVD_OK;
#else
  (void)dev_ptr; (void)bytes;
  return WSVD_E_UNSUPPORTED;      // the product build carries no stamps
#endif
}

wsvd_status wsvd_probe_stream_read(wsvd_ctx* ctx, const void* ptr, size_t bytes, int32_t workgroups, void* hip_stream) {
  if (!ctx || !ptr) return WSVD_E_NULL;
  if (!aligned16(ptr)) return WSVD_E_ALIGN;
  if (bytes < 16 || workgroups < 1 || workgroups > (1 << 20)) return WSVD_E_SHAPE;
  hipError_t e = wsvd_launch_stream_read(ptr, bytes, workgroups, nullptr, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_quantize_act_i8(wsvd_ctx* ctx, const void* x, int32_t x_dtype, int64_t rows, int64_t cols, int8_t* codes,
                                 void* scale_f16, void* hip_stream) {
  if (!ctx || !x || !codes || !scale_f16) return WSVD_E_NULL;
  if (x_dtype != WSVD_F32 && x_dtype != WSVD_BF16) return WSVD_E_DTYPE;
  if (rows < 0 || cols <= 0) return WSVD_E_SHAPE;
  hipError_t e = wsvd_launch_quantize_act_i8(x, x_dtype, rows, cols, codes, scale_f16, (hipStream_t)hip_stream);
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

static wsvd_status linear_w4a8(wsvd_ctx* ctx, const int8_t* x, const void* x_scale, const void* w_i4, const void* w_scale_f16,
                               int64_t M, int64_t K, int64_t N, void* out, int64_t n_first, void* out2, int32_t out_dtype,
                               void* hip_stream) {
  if (!ctx || !x || !x_scale || !w_i4 || !w_scale_f16 || !out) return WSVD_E_NULL;
  if (n_first < N && !out2) return WSVD_E_NULL;
  if (out_dtype != WSVD_F32) return WSVD_E_DTYPE;
  if (M <= 0 || M > 64 || K <= 0 || K % 64 != 0 || K > 65536 || N <= 0 || N % 32 != 0 || M * N > INT32_MAX) return WSVD_E_SHAPE;
  if (n_first <= 0 || n_first > N || n_first % 32 != 0) return WSVD_E_SHAPE;
  if (!aligned16(x) || !aligned16(w_i4) || !aligned16(out) || !aligned16(out2)) return WSVD_E_ALIGN;
  hipError_t e = wsvd_launch_linear_w4a8(x, x_scale, w_i4, w_scale_f16, M, K, N, (float*)out, n_first, (float*)out2,
                                         ctx->opt.linear_direct != 0, (hipStream_t)hip_stream);
  if (e == hipErrorNotSupported) return WSVD_E_UNSUPPORTED;
  return e == hipSuccess ? WSVD_OK : WSVD_E_HIP;
}

wsvd_status wsvd_linear_w4a8(wsvd_ctx* ctx, const int8_t* x, const void* x_scale, const void* w_i4, const void* w_scale_f16,
                             int64_t M, int64_t K, int64_t N, void* out, int32_t out_dtype, void* hip_stream) {
  return linear_w4a8(ctx, x, x_scale, w_i4, w_scale_f16, M, K, N, out, N, nullptr, out_dtype, hip_stream);
}

wsvd_status wsvd_linear_w4a8_split(wsvd_ctx* ctx, const int8_t* x, const void* x_scale, const void* w_i4,
                                   const void* w_scale_f16, int64_t M, int64_t K, int64_t N, int64_t n_first, void* out_first,
                                   void* out_rest, int32_t out_dtype, void* hip_stream) {
  return linear_w4a8(ctx, x, x_scale, w_i4, w_scale_f16, M, K, N, out_first, n_first, out_rest, out_dtype, hip_stream);
}

}  // extern "C"

// ---------------------------------------------------------------- attention launch policy
// Fills the kernel parameters and decides the decomposition: grid = (Hkv, n_chunks, B), threads per workgroup.
void wsvd_attn_plan(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* q, const void* q_scale, const void* B_K,
                    const void* B_V, const wsvd_cache& cache, int max_seq_len, void* out, AttnParams& p, dim3& grid,
                    int& threads, int force_threads) {
  p = AttnParams{};
  p.q = q; p.q_scale = (const uint16_t*)q_scale; p.BK = B_K; p.BV = B_V;
  p.k_codes = (const uint8_t*)cache.k_codes; p.v_codes = (const uint8_t*)cache.v_codes;
  p.k_meta = (const uint16_t*)cache.k_meta; p.v_meta = (const uint16_t*)cache.v_meta;
  p.seq_lens = cache.seq_lens;
  p.out = (float*)out;
  p.tickets = (int*)ctx->ws;
  p.partials = (unsigned long long*)((char*)ctx->ws + (size_t)kWsCounterInts * 4);
  p.err_word = ctx->err_word;
  p.B = d.batch; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads; p.d = d.d_head;
  p.out_dim = d.d_head;
  p.out_bf16 = d.out_dtype == WSVD_BF16;
  p.t_cap = d.t_cap;
  p.q_dtype = d.q_dtype; p.factor_dtype = d.factor_dtype;
  const float sm = d.sm_scale != 0.f ? d.sm_scale : 1.0f / sqrtf((float)d.d_head);
  p.c_scale = sm * kLog2e;
  // Work decomposition.  One unit = one (sequence, kv head) stream.  The grid should put about 16 wavefronts on
  // every CU.  Wavefronts are cheapest to add inside a workgroup (merge through LDS), so the workgroup grows first
  // (MFMA kernels: up to their launch bound); only then is the context split over several workgroups, whose partial
  // results are merged by the last one to finish.  A chunk is a multiple of 64 rows, at least min_chunk (>= 256).
  const int n_units = d.batch * d.n_kv_heads;
  const int max_rows = ((max_seq_len > 0 ? max_seq_len : 1) + 63) / 64 * 64;
  const bool mfma = !(d.latent_dtype == WSVD_F32 || d.latent_dtype == WSVD_BF16);
  // "wg_per_cu" scales the target: 4 (default) = as many wavefronts as fit on the chip at once (the generic kernels
  // and the rank-32 matrix-core kernels hold 16 per CU, the rank-64 ones 8), so that the grid runs in a single round:
  // a second round pays the prologue, the split merge and the B_V epilogue again with the memory system idle
  const int resident = mfma ? wsvd_attn_mfma_waves_per_cu(d.latent_dtype, d.rank, p.G) : 16;
  const int waves_target = ctx->n_cu * resident * ctx->opt.wg_per_cu / 4;
  int waves_per_unit = (waves_target + n_units - 1) / n_units;
  const int max_tiles = max_rows / 64;
  if (waves_per_unit > max_tiles) waves_per_unit = max_tiles;
  int nw = 4;
  if (mfma) {
    const int bound = wsvd_attn_mfma_max_threads(d.latent_dtype, d.rank, p.G);
    const int nw_max = (ctx->opt.max_threads && ctx->opt.max_threads < bound ? ctx->opt.max_threads : bound) / 64;
    while (nw * 2 <= nw_max && nw * 2 <= waves_per_unit) nw *= 2;
    if (force_threads) nw = force_threads / 64;     // the fused step: one workgroup size for both roles
  }
  int chunks_wanted = waves_per_unit / nw;
  if (chunks_wanted < 1) chunks_wanted = 1;
  int chunk_rows = ((max_rows + chunks_wanted - 1) / chunks_wanted + 63) / 64 * 64;
  const bool auto_chunk = ctx->opt.min_chunk == 0;          // no explicit setting: the policy below may also undo a split
  int min_chunk = ctx->opt.min_chunk < 256 ? 256 : ctx->opt.min_chunk;
  // fp32 / bf16 latents (4-wave workgroups, single sequences in practice): a second chunk costs a hand-off between
  // workgroups (about 3 us) and saves half a chunk's stream; below 1024 rows per chunk that is a loss (640 rows of bf16
  // latents: 9.2 us as two chunks, 8.3 us as one)
  if (!mfma && min_chunk < 1024) min_chunk = 1024;
  if (chunk_rows < min_chunk) chunk_rows = min_chunk;
  p.chunk_rows = chunk_rows;
  p.n_chunks = (max_rows + chunk_rows - 1) / chunk_rows;
  // A split costs a hand-off between workgroups at the end (2.6 us measured) and saves part of one workgroup's stream
  // (about 60 GB/s: 2.35 us for the 139 KB of a 2048-row rank-32 int8 unit).  With at most one unit per two compute units
  // and below about 300 KB per (sequence, kv head) no split pays: 1 to 4 sequences of 32 heads and 2048 rows take
  // 7.8-9.0 us as one chunk and 9.4-10.7 us as two; from 8 sequences on the two are level, at 12 the split wins by 0.7 us.
  if (auto_chunk && mfma && p.n_chunks > 1 && n_units * 2 <= ctx->n_cu &&
      (size_t)max_rows * 2 * (size_t)(row_bytes_host(d) + meta_bytes_host(d)) < (size_t)300 * 1024) {
    p.chunk_rows = (max_rows + 63) / 64 * 64;
    p.n_chunks = 1;
  }
  grid = dim3((unsigned)d.n_kv_heads, (unsigned)p.n_chunks, (unsigned)d.batch);
  threads = nw * 64;
  const size_t tl_need = (size_t)grid.x * grid.y * grid.z * kTimelineWaves * kTimelineSlots * sizeof(long long);
  p.timeline = (ctx->timeline && ctx->timeline_bytes >= tl_need) ? ctx->timeline : nullptr;
}

// bytes of split words the launch wsvd_attn_plan chooses for this call touches
size_t wsvd_attn_split_bytes(const wsvd_ctx* ctx, const wsvd_layer_desc& d, int max_seq_len) {
  AttnParams p;
  dim3 grid;
  int threads;
  wsvd_attn_plan(ctx, d, nullptr, nullptr, nullptr, nullptr, wsvd_cache{}, max_seq_len, nullptr, p, grid, threads, 0);
  const size_t vec = (size_t)(d.rank > d.d_head ? d.rank : d.d_head) + 2;
  return p.n_chunks > 1 ? (size_t)d.batch * d.n_q_heads * p.n_chunks * vec * 8 : 0;
}

hipError_t wsvd_launch_attn(const wsvd_ctx* ctx, const wsvd_layer_desc& d, const void* q, const void* q_scale,
                            const void* B_K, const void* B_V, const wsvd_cache& cache, int max_seq_len, void* out,
                            hipStream_t s) {
  AttnParams p;
  dim3 grid;
  int threads;
  wsvd_attn_plan(ctx, d, q, q_scale, B_K, B_V, cache, max_seq_len, out, p, grid, threads, 0);
  const bool mfma = !(d.latent_dtype == WSVD_F32 || d.latent_dtype == WSVD_BF16);
  if (!mfma) return wsvd_launch_attn_generic(p, d.latent_dtype, d.rank, grid, s);
  return wsvd_launch_attn_mfma(p, d.latent_dtype, d.rank, grid, threads, s);
}
