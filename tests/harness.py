"""Glue for the GPU parity tests: moves oracle-side (numpy, logical format) data to the device through
the library's own import / export entry points and wraps the calls.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

import oracle as O
import paper_2604_02570_amd as W


def dev(arr: np.ndarray) -> torch.Tensor:
    """numpy -> cuda tensor of the same bytes (uint16 / float16 patterns travel as int16)."""
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def bf16_dev(x32: np.ndarray) -> torch.Tensor:
    """fp32 values that are exactly representable in bf16 -> device bf16 bit patterns."""
    bits = (np.ascontiguousarray(x32, np.float32).view(np.uint32) >> 16).astype(np.uint16)
    assert ((bits.astype(np.uint32) << 16).view(np.float32) == x32).all(), "value not bf16-exact"
    return dev(bits)


def as_dtype_dev(x32: np.ndarray, dtype: str) -> torch.Tensor:
    return bf16_dev(x32) if dtype == "bf16" else dev(np.ascontiguousarray(x32, np.float32))


class DeviceLayer:
    """A layer's device-side state: context, descriptor, cache planes, workspace."""

    def __init__(self, batch, n_q_heads, n_kv_heads, d_head, d_model, rank, t_cap, latent_dtype, factor_dtype,
                 x_dtype, q_dtype, sm_scale=0.0, poison=True):
        self.desc = W.layer_desc(batch, n_q_heads, n_kv_heads, d_head, d_model, rank, t_cap, latent_dtype, factor_dtype,
                                 x_dtype, q_dtype, "f32", sm_scale)
        self.latent_dtype = latent_dtype
        self.B, self.Hq, self.Hkv, self.d, self.E, self.r, self.t_cap = batch, n_q_heads, n_kv_heads, d_head, d_model, rank, t_cap
        self.ctx = W.wsvd_create(0)
        cb, mb = W.wsvd_cache_bytes(self.desc)
        fill = 0xA5 if poison else 0           # garbage in never-written rows must not leak into results
        self.k_codes = torch.full((cb,), fill, dtype=torch.uint8, device="cuda")
        self.v_codes = torch.full((cb,), fill, dtype=torch.uint8, device="cuda")
        self.k_meta = torch.full((max(mb, 16),), 0xFF if poison else 0, dtype=torch.uint8, device="cuda")  # fp16 NaN pattern
        self.v_meta = torch.full((max(mb, 16),), 0xFF if poison else 0, dtype=torch.uint8, device="cuda")
        self.seq_lens = torch.zeros(batch, dtype=torch.int32, device="cuda")
        self.cache = W.make_cache(self.k_codes, self.v_codes, self.k_meta, self.v_meta, self.seq_lens)
        self.ws = torch.empty(W.wsvd_workspace_bytes(self.desc), dtype=torch.uint8, device="cuda")
        W.wsvd_set_workspace(self.ctx, self.ws)
        self.out = torch.full((batch, n_q_heads, d_head), float("nan"), dtype=torch.float32, device="cuda")

    def close(self):
        torch.cuda.synchronize()
        W.wsvd_destroy(self.ctx)

    # ---- oracle cache (logical) -> device layout
    def upload(self, oc: O.LatentCache, n_rows=None):
        n_rows = n_rows or oc.t_cap
        for plane, codes, scale, zero in ((0, oc.k, oc.k_scale, oc.k_zero), (1, oc.v, oc.v_scale, oc.v_zero)):
            lc = dev(codes[:, :, :n_rows])
            meta = None
            if oc.dtype == "i8":
                meta = dev(scale[:, :, :n_rows].view(np.uint16))
            elif oc.dtype == "i4":
                meta = dev(np.stack([scale[:, :, :n_rows].view(np.uint16), zero[:, :, :n_rows].view(np.uint16)], axis=-1))
            W.wsvd_cache_import(self.ctx, self.desc, plane, lc, meta, 0, n_rows, self.cache)
        self.seq_lens.copy_(torch.from_numpy(oc.seq_lens.astype(np.int32)))
        torch.cuda.synchronize()

    # ---- device layout -> logical numpy (codes, scale, zero) for rows [t0, t0+n)
    def download(self, plane, t0, n):
        rb = {"f32": self.r * 4, "bf16": self.r * 2, "i8": self.r, "i4": self.r // 2}[self.latent_dtype]
        lc = torch.zeros((self.B, self.Hkv, n, rb), dtype=torch.uint8, device="cuda")
        per = {"i8": 1, "i4": 2}.get(self.latent_dtype, 0)
        meta = torch.zeros((self.B, self.Hkv, n, max(per, 1)), dtype=torch.int16, device="cuda")
        W.wsvd_cache_export(self.ctx, self.desc, plane, self.cache, t0, n, lc, meta if per else None)
        torch.cuda.synchronize()
        raw = lc.cpu().numpy()
        m = meta.cpu().numpy().view(np.uint16)
        if self.latent_dtype == "f32":
            return raw.view(np.float32), None, None
        if self.latent_dtype == "bf16":
            return raw.view(np.uint16), None, None
        if self.latent_dtype == "i8":
            return raw.view(np.int8), m[..., 0].view(np.float16), None
        return raw, m[..., 0].view(np.float16), m[..., 1].view(np.float16)

    def attend(self, q_dev, q_scale_dev, BK_dev, BV_dev, max_seq_len):
        self.out.fill_(float("nan"))
        W.wsvd_decode_attn(self.ctx, self.desc, q_dev, q_scale_dev, BK_dev, BV_dev, self.cache, max_seq_len, self.out)
        st = W.wsvd_check(self.ctx)
        assert st == 0, W.status_str(st)
        return self.out.cpu().numpy().astype(np.float64)

    def attend_rope(self, q_dev, q_scale_dev, BK_dev, BV_dev, max_seq_len, rope_base):
        self.out.fill_(float("nan"))
        W.wsvd_decode_attn_rope(self.ctx, self.desc, q_dev, q_scale_dev, BK_dev, BV_dev, self.cache, max_seq_len, rope_base,
                                self.out)
        st = W.wsvd_check(self.ctx)
        assert st == 0, W.status_str(st)
        return self.out.cpu().numpy().astype(np.float64)

    def pack_A(self, A32: np.ndarray, dtype: str) -> torch.Tensor:
        """Down-projection factor [Hkv,E,r] (the paper's shape, row-major) -> the library's packed layout."""
        src = as_dtype_dev(A32, dtype)
        dst = torch.empty(W.wsvd_factor_a_bytes(self.desc), dtype=torch.uint8, device="cuda")
        W.wsvd_pack_factor_a(self.ctx, self.desc, src, dst)
        torch.cuda.synchronize()
        return dst

    def step(self, x_dev, AK_dev, AV_dev, q_dev, q_scale_dev, BK_dev, BV_dev, max_seq_len):
        """wsvd_decode_step; returns (output, device status word)."""
        self.out.fill_(float("nan"))
        W.wsvd_decode_step(self.ctx, self.desc, x_dev, None, AK_dev, AV_dev, q_dev, q_scale_dev, BK_dev, BV_dev, self.cache,
                           max_seq_len, self.out)
        st = W.wsvd_check(self.ctx)
        return self.out.cpu().numpy().astype(np.float64), st

    def append(self, x_dev, x_scale_dev, AK_dev, AV_dev):
        W.wsvd_latent_append(self.ctx, self.desc, x_dev, x_scale_dev, AK_dev, AV_dev, self.cache)
        return W.wsvd_check(self.ctx)


def q_to_device(q32: np.ndarray, q_dtype: str):
    """Query [B,Hq,d] fp32 -> (device tensor, device scale or None, fp64 value the oracle must use).
    int8 queries are produced by the ORACLE's per-token quantiser (one scale per token over all heads)."""
    B = q32.shape[0]
    if q_dtype == "i8":
        codes, s = O.quantize_act_i8(q32.reshape(B, -1))
        q64 = (codes.astype(np.float64) * s.astype(np.float64)[:, None]).reshape(q32.shape)
        return dev(codes.reshape(q32.shape)), dev(s.view(np.uint16)), q64
    if q_dtype == "bf16":
        bits = O.bf16_bits_from_f32(q32)
        return dev(bits), None, O.f64_from_bf16_bits(bits)
    return dev(q32.astype(np.float32)), None, q32.astype(np.float32).astype(np.float64)


def err_stats(got: np.ndarray, ref: np.ndarray):
    """(max abs error, max abs error / max |ref|, relative L2)."""
    diff = got - ref
    return float(np.abs(diff).max()), float(np.abs(diff).max() / max(np.abs(ref).max(), 1e-300)), \
        float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))
