"""Thin ctypes binding of libwsvd.so (the gfx950 WSVD decode library).

Argument marshalling only: every step of the decode path runs in the library's HIP kernels.
PyTorch supplies device memory (``tensor.data_ptr()``) and the current HIP stream.  There is no
CPU fallback: if the shared library is missing or a call fails, an exception is raised.
Function names mirror include/wsvd.h.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwsvd.so")

F32, BF16, F16, I8, I4 = 0, 1, 2, 3, 4
DTYPES = {"f32": F32, "bf16": BF16, "f16": F16, "i8": I8, "i4": I4}

STATUS_NAMES = {0: "WSVD_OK", 1: "WSVD_E_NULL", 2: "WSVD_E_SHAPE", 3: "WSVD_E_DTYPE", 4: "WSVD_E_ALIGN",
                5: "WSVD_E_CAPACITY", 6: "WSVD_E_UNSUPPORTED", 7: "WSVD_E_HIP", 8: "WSVD_E_WORKSPACE"}

OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_CAPACITY, E_UNSUPPORTED, E_HIP, E_WORKSPACE = range(9)

# every symbol include/wsvd.h declares
EXPORTS = ["wsvd_create", "wsvd_destroy", "wsvd_cache_bytes", "wsvd_workspace_bytes", "wsvd_set_workspace",
           "wsvd_ctx_set_option", "wsvd_latent_append", "wsvd_latent_store", "wsvd_decode_attn", "wsvd_decode_attn_store", "wsvd_decode_attn_static",
           "wsvd_paged_cache_bytes", "wsvd_latent_append_paged", "wsvd_prefill_append_paged", "wsvd_prefill_attn_paged", "wsvd_decode_attn_paged", "wsvd_decode_attn_rope", "wsvd_decode_step", "wsvd_check", "wsvd_status_str",
           "wsvd_factor_a_bytes", "wsvd_pack_factor_a", "wsvd_quantize_rows", "wsvd_cache_import", "wsvd_cache_export", "wsvd_quantize_act_i8", "wsvd_linear_w4a8",
           "wsvd_linear_w4a8_split", "wsvd_probe_stream_read", "wsvd_test_step_attention", "wsvd_fold_qk", "wsvd_fold_vo", "wsvd_decode_attn_latent",
           "wsvd_rmsnorm_quant_i8", "wsvd_swiglu_quant_i8", "wsvd_prefill_append",
           "wsvd_prefill_attn", "wsvd_shared_workspace_bytes", "wsvd_decode_attn_shared", "wsvd_timeline_set_buffer"]


class WsvdError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_str(status)})")


class LayerDesc(ctypes.Structure):
    _fields_ = [("batch", c_int32), ("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("d_head", c_int32),
                ("d_model", c_int32), ("rank", c_int32), ("t_cap", c_int32), ("latent_dtype", c_int32),
                ("factor_dtype", c_int32), ("x_dtype", c_int32), ("q_dtype", c_int32), ("out_dtype", c_int32),
                ("sm_scale", c_float)]


class Cache(ctypes.Structure):
    _fields_ = [("k_codes", c_void_p), ("v_codes", c_void_p), ("k_meta", c_void_p), ("v_meta", c_void_p),
                ("seq_lens", c_void_p)]


class PagedCache(ctypes.Structure):
    _fields_ = [("k_codes", c_void_p), ("v_codes", c_void_p), ("k_meta", c_void_p), ("v_meta", c_void_p),
                ("seq_lens", c_void_p), ("block_table", c_void_p), ("page_rows", c_int32), ("max_pages", c_int32),
                ("n_pages", c_int32)]


_lib = None


def use_library(path: str):
    """Load another build of the library (the profiling build libwsvd_timeline.so) instead of libwsvd.so.  Must be
    called before the first call into the library."""
    global LIB_PATH
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    if not os.path.exists(path):
        raise FileNotFoundError(path)
    LIB_PATH = path


def lib():
    """Load libwsvd.so (built by paper_2604_02570_amd.build / __graft_entry__.build).  Fails loudly."""
    global _lib
    if _lib is None:
        # PyTorch brings its own copy of the HIP runtime: it has to be loaded before this library pulls in the system's,
        # or device calls made through the second copy fail
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            # nothing built yet: build in-tree once; a failed build raises (there is no fallback path)
            from .build import build
            build(verbose=False)
        L = ctypes.CDLL(LIB_PATH)
        L.wsvd_status_str.restype = c_char_p
        L.wsvd_status_str.argtypes = [c_int]
        L.wsvd_create.argtypes = [POINTER(c_void_p), c_int]
        L.wsvd_destroy.argtypes = [c_void_p]
        L.wsvd_cache_bytes.argtypes = [POINTER(LayerDesc), POINTER(c_size_t), POINTER(c_size_t)]
        L.wsvd_workspace_bytes.argtypes = [POINTER(LayerDesc), POINTER(c_size_t)]
        L.wsvd_set_workspace.argtypes = [c_void_p, c_void_p, c_size_t]
        L.wsvd_ctx_set_option.argtypes = [c_void_p, c_char_p, c_int]
        L.wsvd_latent_append.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_void_p, c_void_p,
                                         POINTER(Cache), c_void_p]
        L.wsvd_latent_store.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_int64, POINTER(Cache), c_void_p]
        L.wsvd_decode_attn.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_void_p, c_void_p,
                                       POINTER(Cache), c_int32, c_void_p, c_void_p]
        L.wsvd_decode_attn_static.argtypes = L.wsvd_decode_attn.argtypes
        L.wsvd_test_step_attention.argtypes = L.wsvd_decode_attn.argtypes
        L.wsvd_paged_cache_bytes.argtypes = [POINTER(LayerDesc), c_int32, c_int32, POINTER(c_size_t), POINTER(c_size_t)]
        L.wsvd_latent_append_paged.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_void_p, c_void_p,
                                               POINTER(PagedCache), c_void_p]
        L.wsvd_prefill_attn_paged.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_int32, c_int32, c_void_p, c_void_p,
                                              POINTER(PagedCache), c_int32, c_void_p, c_void_p]
        L.wsvd_prefill_append_paged.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_int32, c_int32, c_void_p, c_void_p,
                                                POINTER(PagedCache), c_void_p]
        L.wsvd_decode_attn_paged.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_void_p, c_void_p,
                                             POINTER(PagedCache), c_int32, c_void_p, c_void_p]
        L.wsvd_decode_attn_store.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_int64, c_void_p, c_void_p, c_void_p,
                                             c_void_p, POINTER(Cache), c_int32, c_void_p, c_void_p]
        L.wsvd_decode_attn_rope.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_void_p, c_void_p,
                                            POINTER(Cache), c_int32, c_float, c_void_p, c_void_p]
        L.wsvd_decode_step.argtypes = [c_void_p, POINTER(LayerDesc)] + [c_void_p] * 8 + [POINTER(Cache), c_int32, c_void_p, c_void_p]
        L.wsvd_check.argtypes = [c_void_p, c_void_p]
        L.wsvd_factor_a_bytes.argtypes = [POINTER(LayerDesc), POINTER(c_size_t)]
        L.wsvd_pack_factor_a.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_void_p]
        L.wsvd_quantize_rows.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_int64, c_void_p, c_void_p, c_void_p]
        L.wsvd_cache_import.argtypes = [c_void_p, POINTER(LayerDesc), c_int32, c_void_p, c_void_p, c_int32, c_int32,
                                        POINTER(Cache), c_void_p]
        L.wsvd_cache_export.argtypes = [c_void_p, POINTER(LayerDesc), c_int32, POINTER(Cache), c_int32, c_int32,
                                        c_void_p, c_void_p, c_void_p]
        L.wsvd_quantize_act_i8.argtypes = [c_void_p, c_void_p, c_int32, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
        L.wsvd_linear_w4a8.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64,
                                       c_void_p, c_int32, c_void_p]
        L.wsvd_linear_w4a8_split.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64,
                                             c_int64, c_void_p, c_void_p, c_int32, c_void_p]
        L.wsvd_timeline_set_buffer.argtypes = [c_void_p, c_void_p, c_size_t]
        L.wsvd_probe_stream_read.argtypes = [c_void_p, c_void_p, c_size_t, c_int32, c_void_p]
        L.wsvd_prefill_append.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p,
                                          POINTER(Cache), c_void_p]
        L.wsvd_prefill_attn.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_int32, c_int32, c_void_p, c_void_p, POINTER(Cache),
                                        c_int32, c_void_p, c_void_p]
        L.wsvd_shared_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, c_int32, c_int32, POINTER(c_size_t)]
        L.wsvd_decode_attn_shared.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_int32, c_int32, c_float] + [c_void_p] * 9 + \
                                             [c_size_t, c_void_p, c_void_p]
        L.wsvd_fold_qk.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_int32, c_void_p, c_void_p, c_void_p]
        L.wsvd_fold_vo.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_void_p, c_void_p, c_void_p]
        L.wsvd_decode_attn_latent.argtypes = [c_void_p, POINTER(LayerDesc), c_void_p, c_int32, c_void_p, POINTER(Cache), c_int32,
                                              c_void_p, c_void_p]
        L.wsvd_rmsnorm_quant_i8.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_float, c_int64, c_int64, c_void_p,
                                            c_void_p, c_void_p, c_void_p]
        L.wsvd_swiglu_quant_i8.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
        for name in EXPORTS:
            if name not in ("wsvd_status_str",):
                getattr(L, name).restype = c_int
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().wsvd_status_str(int(status)).decode()


def _ck(status, where):
    if status != 0:
        raise WsvdError(status, where)


def _ptr(t):
    """Device (or host) address of a torch tensor, None -> NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return c_void_p(t)
    return c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return c_void_p(stream)
    return c_void_p(stream.cuda_stream)


def layer_desc(batch, n_q_heads, n_kv_heads, d_head, d_model, rank, t_cap, latent_dtype, factor_dtype, x_dtype,
               q_dtype, out_dtype="f32", sm_scale=0.0) -> LayerDesc:
    g = lambda v: DTYPES[v] if isinstance(v, str) else int(v)
    return LayerDesc(batch, n_q_heads, n_kv_heads, d_head, d_model, rank, t_cap, g(latent_dtype), g(factor_dtype),
                     g(x_dtype), g(q_dtype), g(out_dtype), float(sm_scale))


def wsvd_create(device_ordinal: int = 0):
    h = c_void_p()
    _ck(lib().wsvd_create(byref(h), device_ordinal), "wsvd_create")
    return h


def wsvd_destroy(ctx):
    _ck(lib().wsvd_destroy(ctx), "wsvd_destroy")


def wsvd_cache_bytes(desc):
    a, b = c_size_t(), c_size_t()
    _ck(lib().wsvd_cache_bytes(byref(desc), byref(a), byref(b)), "wsvd_cache_bytes")
    return a.value, b.value


def wsvd_workspace_bytes(desc):
    a = c_size_t()
    _ck(lib().wsvd_workspace_bytes(byref(desc), byref(a)), "wsvd_workspace_bytes")
    return a.value


def wsvd_set_workspace(ctx, ws_tensor):
    _ck(lib().wsvd_set_workspace(ctx, _ptr(ws_tensor), ws_tensor.numel() * ws_tensor.element_size()), "wsvd_set_workspace")


def wsvd_ctx_set_option(ctx, name: str, value: int):
    _ck(lib().wsvd_ctx_set_option(ctx, name.encode(), int(value)), "wsvd_ctx_set_option")


def wsvd_factor_a_bytes(desc):
    a = c_size_t()
    _ck(lib().wsvd_factor_a_bytes(byref(desc), byref(a)), "wsvd_factor_a_bytes")
    return a.value


def wsvd_pack_factor_a(ctx, desc, A_row_major, A_packed, stream=None):
    _ck(lib().wsvd_pack_factor_a(ctx, byref(desc), _ptr(A_row_major), _ptr(A_packed), _stream(stream)), "wsvd_pack_factor_a")


def make_cache(k_codes, v_codes, k_meta, v_meta, seq_lens) -> Cache:
    c = Cache(_ptr(k_codes), _ptr(v_codes), _ptr(k_meta), _ptr(v_meta), _ptr(seq_lens))
    c._keep = (k_codes, v_codes, k_meta, v_meta, seq_lens)   # keep the tensors alive
    return c


def wsvd_latent_append(ctx, desc, x, x_scale, A_K, A_V, cache, stream=None):
    _ck(lib().wsvd_latent_append(ctx, byref(desc), _ptr(x), _ptr(x_scale), _ptr(A_K), _ptr(A_V), byref(cache),
                                 _stream(stream)), "wsvd_latent_append")


def wsvd_latent_store(ctx, desc, c_K, c_V, ld, cache, stream=None):
    _ck(lib().wsvd_latent_store(ctx, byref(desc), _ptr(c_K), _ptr(c_V), int(ld), byref(cache), _stream(stream)),
        "wsvd_latent_store")


def wsvd_decode_attn(ctx, desc, q, q_scale, B_K, B_V, cache, max_seq_len, out, stream=None):
    _ck(lib().wsvd_decode_attn(ctx, byref(desc), _ptr(q), _ptr(q_scale), _ptr(B_K), _ptr(B_V), byref(cache),
                               int(max_seq_len), _ptr(out), _stream(stream)), "wsvd_decode_attn")


def wsvd_test_step_attention(ctx, desc, q, q_scale, B_K, B_V, cache, max_seq_len, out, stream=None):
    """Measurement aid (include/wsvd_test.h): the second launch of the last deferred-row wsvd_decode_step, once more."""
    _ck(lib().wsvd_test_step_attention(ctx, byref(desc), _ptr(q), _ptr(q_scale), _ptr(B_K), _ptr(B_V), byref(cache),
                                       int(max_seq_len), _ptr(out), _stream(stream)), "wsvd_test_step_attention")


def wsvd_decode_attn_store(ctx, desc, c_K, c_V, ld, q, q_scale, B_K, B_V, cache, max_seq_len, out, stream=None):
    _ck(lib().wsvd_decode_attn_store(ctx, byref(desc), _ptr(c_K), _ptr(c_V), int(ld), _ptr(q), _ptr(q_scale), _ptr(B_K), _ptr(B_V),
                                     byref(cache), int(max_seq_len), _ptr(out), _stream(stream)), "wsvd_decode_attn_store")


def make_paged_cache(k_codes, v_codes, k_meta, v_meta, seq_lens, block_table, page_rows, max_pages, n_pages) -> PagedCache:
    c = PagedCache(_ptr(k_codes), _ptr(v_codes), _ptr(k_meta), _ptr(v_meta), _ptr(seq_lens), _ptr(block_table),
                   int(page_rows), int(max_pages), int(n_pages))
    c._keep = (k_codes, v_codes, k_meta, v_meta, seq_lens, block_table)   # keep the tensors alive
    return c


def wsvd_paged_cache_bytes(desc, page_rows, n_pages):
    a, b = c_size_t(), c_size_t()
    _ck(lib().wsvd_paged_cache_bytes(byref(desc), int(page_rows), int(n_pages), byref(a), byref(b)), "wsvd_paged_cache_bytes")
    return a.value, b.value


def wsvd_latent_append_paged(ctx, desc, x, x_scale, A_K, A_V, cache, stream=None):
    _ck(lib().wsvd_latent_append_paged(ctx, byref(desc), _ptr(x), _ptr(x_scale), _ptr(A_K), _ptr(A_V), byref(cache),
                                       _stream(stream)), "wsvd_latent_append_paged")


def wsvd_prefill_append_paged(ctx, desc, x, n_tokens, seq_index, A_K, A_V, cache, stream=None):
    _ck(lib().wsvd_prefill_append_paged(ctx, byref(desc), _ptr(x), int(n_tokens), int(seq_index), _ptr(A_K), _ptr(A_V), byref(cache),
                                        _stream(stream)), "wsvd_prefill_append_paged")


def wsvd_prefill_attn_paged(ctx, desc, q, n_q, n_after, B_K, B_V, cache, max_seq_len, out, stream=None):
    _ck(lib().wsvd_prefill_attn_paged(ctx, byref(desc), _ptr(q), int(n_q), int(n_after), _ptr(B_K), _ptr(B_V), byref(cache),
                                      int(max_seq_len), _ptr(out), _stream(stream)), "wsvd_prefill_attn_paged")


def wsvd_decode_attn_paged(ctx, desc, q, q_scale, B_K, B_V, cache, max_seq_len, out, stream=None):
    _ck(lib().wsvd_decode_attn_paged(ctx, byref(desc), _ptr(q), _ptr(q_scale), _ptr(B_K), _ptr(B_V), byref(cache),
                                     int(max_seq_len), _ptr(out), _stream(stream)), "wsvd_decode_attn_paged")


def wsvd_decode_attn_static(ctx, desc, q, q_scale, B_K, B_V, cache, max_seq_len, out, stream=None):
    _ck(lib().wsvd_decode_attn_static(ctx, byref(desc), _ptr(q), _ptr(q_scale), _ptr(B_K), _ptr(B_V), byref(cache),
                                      int(max_seq_len), _ptr(out), _stream(stream)), "wsvd_decode_attn_static")


def wsvd_decode_attn_rope(ctx, desc, q, q_scale, B_K, B_V, cache, max_seq_len, rope_base, out, stream=None):
    _ck(lib().wsvd_decode_attn_rope(ctx, byref(desc), _ptr(q), _ptr(q_scale), _ptr(B_K), _ptr(B_V), byref(cache),
                                    int(max_seq_len), float(rope_base), _ptr(out), _stream(stream)), "wsvd_decode_attn_rope")


def wsvd_decode_step(ctx, desc, x, x_scale, A_K, A_V, q, q_scale, B_K, B_V, cache, max_seq_len, out, stream=None):
    _ck(lib().wsvd_decode_step(ctx, byref(desc), _ptr(x), _ptr(x_scale), _ptr(A_K), _ptr(A_V), _ptr(q), _ptr(q_scale),
                               _ptr(B_K), _ptr(B_V), byref(cache), int(max_seq_len), _ptr(out), _stream(stream)),
        "wsvd_decode_step")


def wsvd_check(ctx, stream=None) -> int:
    """Synchronise and return the device-side status word (0 = ok)."""
    return lib().wsvd_check(ctx, _stream(stream))


def wsvd_quantize_rows(ctx, desc, c, n_rows, codes, meta, stream=None):
    _ck(lib().wsvd_quantize_rows(ctx, byref(desc), _ptr(c), int(n_rows), _ptr(codes), _ptr(meta), _stream(stream)),
        "wsvd_quantize_rows")


def wsvd_cache_import(ctx, desc, which_plane, codes, meta, t0, n_rows, cache, stream=None):
    _ck(lib().wsvd_cache_import(ctx, byref(desc), int(which_plane), _ptr(codes), _ptr(meta), int(t0), int(n_rows),
                                byref(cache), _stream(stream)), "wsvd_cache_import")


def wsvd_cache_export(ctx, desc, which_plane, cache, t0, n_rows, codes, meta, stream=None):
    _ck(lib().wsvd_cache_export(ctx, byref(desc), int(which_plane), byref(cache), int(t0), int(n_rows), _ptr(codes),
                                _ptr(meta), _stream(stream)), "wsvd_cache_export")


def wsvd_quantize_act_i8(ctx, x, x_dtype, rows, cols, codes, scale, stream=None):
    dt = DTYPES[x_dtype] if isinstance(x_dtype, str) else int(x_dtype)
    _ck(lib().wsvd_quantize_act_i8(ctx, _ptr(x), dt, int(rows), int(cols), _ptr(codes), _ptr(scale), _stream(stream)),
        "wsvd_quantize_act_i8")


def wsvd_linear_w4a8(ctx, x, x_scale, w_i4, w_scale, M, K, N, out, stream=None):
    _ck(lib().wsvd_linear_w4a8(ctx, _ptr(x), _ptr(x_scale), _ptr(w_i4), _ptr(w_scale), int(M), int(K), int(N),
                               _ptr(out), F32, _stream(stream)), "wsvd_linear_w4a8")


def wsvd_prefill_append(ctx, desc, x, x_scale, n_tokens, seq_index, A_K, A_V, cache, stream=None):
    _ck(lib().wsvd_prefill_append(ctx, byref(desc), _ptr(x), _ptr(x_scale), int(n_tokens), int(seq_index), _ptr(A_K), _ptr(A_V),
                                  byref(cache), _stream(stream)), "wsvd_prefill_append")


def wsvd_prefill_attn(ctx, desc, q, n_q, n_after, B_K, B_V, cache, max_seq_len, out, stream=None):
    _ck(lib().wsvd_prefill_attn(ctx, byref(desc), _ptr(q), int(n_q), int(n_after), _ptr(B_K), _ptr(B_V), byref(cache),
                                int(max_seq_len), _ptr(out), _stream(stream)), "wsvd_prefill_attn")


def wsvd_shared_workspace_bytes(batch, n_heads, d_head, rank, t_cap):
    a = c_size_t()
    _ck(lib().wsvd_shared_workspace_bytes(int(batch), int(n_heads), int(d_head), int(rank), int(t_cap), byref(a)),
        "wsvd_shared_workspace_bytes")
    return a.value


def wsvd_decode_attn_shared(ctx, batch, n_heads, d_head, rank, t_cap, sm_scale, q, B_K, B_V, k_codes, v_codes, k_scale, v_scale,
                            seq_lens, workspace, out, stream=None):
    _ck(lib().wsvd_decode_attn_shared(ctx, int(batch), int(n_heads), int(d_head), int(rank), int(t_cap), float(sm_scale), _ptr(q),
                                      _ptr(B_K), _ptr(B_V), _ptr(k_codes), _ptr(v_codes), _ptr(k_scale), _ptr(v_scale),
                                      _ptr(seq_lens), _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(out),
                                      _stream(stream)), "wsvd_decode_attn_shared")


def wsvd_fold_qk(ctx, desc, B_Q, rq, B_K, out, stream=None):
    _ck(lib().wsvd_fold_qk(ctx, byref(desc), _ptr(B_Q), int(rq), _ptr(B_K), _ptr(out), _stream(stream)), "wsvd_fold_qk")


def wsvd_fold_vo(ctx, desc, B_V, W_O, out, stream=None):
    _ck(lib().wsvd_fold_vo(ctx, byref(desc), _ptr(B_V), _ptr(W_O), _ptr(out), _stream(stream)), "wsvd_fold_vo")


def wsvd_decode_attn_latent(ctx, desc, c_Q, rq, qk_fold, cache, max_seq_len, u_out, stream=None):
    _ck(lib().wsvd_decode_attn_latent(ctx, byref(desc), _ptr(c_Q), int(rq), _ptr(qk_fold), byref(cache), int(max_seq_len),
                                      _ptr(u_out), _stream(stream)), "wsvd_decode_attn_latent")


def wsvd_rmsnorm_quant_i8(ctx, x, y_add, gain, eps, rows, cols, x_out, codes, scale, stream=None):
    _ck(lib().wsvd_rmsnorm_quant_i8(ctx, _ptr(x), _ptr(y_add), _ptr(gain), float(eps), int(rows), int(cols), _ptr(x_out),
                                    _ptr(codes), _ptr(scale), _stream(stream)), "wsvd_rmsnorm_quant_i8")


def wsvd_swiglu_quant_i8(ctx, gate_up, rows, F, codes, scale, stream=None):
    _ck(lib().wsvd_swiglu_quant_i8(ctx, _ptr(gate_up), int(rows), int(F), _ptr(codes), _ptr(scale), _stream(stream)),
        "wsvd_swiglu_quant_i8")


def wsvd_linear_w4a8_split(ctx, x, x_scale, w_i4, w_scale, M, K, N, n_first, out_first, out_rest, stream=None):
    _ck(lib().wsvd_linear_w4a8_split(ctx, _ptr(x), _ptr(x_scale), _ptr(w_i4), _ptr(w_scale), int(M), int(K), int(N),
                                     int(n_first), _ptr(out_first), _ptr(out_rest), F32, _stream(stream)),
        "wsvd_linear_w4a8_split")


def wsvd_probe_stream_read(ctx, buf, nbytes, workgroups, stream=None):
    _ck(lib().wsvd_probe_stream_read(ctx, _ptr(buf), int(nbytes), int(workgroups), _stream(stream)), "wsvd_probe_stream_read")


def wsvd_timeline_set_buffer(ctx, buf):
    """Profiling build only (include/wsvd_test.h); buf = int64 device tensor or None."""
    n = 0 if buf is None else buf.numel() * buf.element_size()
    _ck(lib().wsvd_timeline_set_buffer(ctx, _ptr(buf), n), "wsvd_timeline_set_buffer")
