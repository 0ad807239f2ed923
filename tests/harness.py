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
                 x_dtype, q_dtype, sm_scale=0.0, poison=True, min_chunk=256):
        self.desc = W.layer_desc(batch, n_q_heads, n_kv_heads, d_head, d_model, rank, t_cap, latent_dtype, factor_dtype,
                                 x_dtype, q_dtype, "f32", sm_scale)
        self.latent_dtype = latent_dtype
        self.B, self.Hq, self.Hkv, self.d, self.E, self.r, self.t_cap = batch, n_q_heads, n_kv_heads, d_head, d_model, rank, t_cap
        self.ctx = W.wsvd_create(0)
        # the tests' small shapes would mostly run as single chunks under the library's automatic policy: chunks of 256
        # rows keep the split paths (hand-off, merge) in play; min_chunk=0 (the full-size cases) = the automatic policy
        W.wsvd_ctx_set_option(self.ctx, "min_chunk", min_chunk)
        cb, mb = W.wsvd_cache_bytes(self.desc)
        # garbage in never-written rows must not leak into results: int codes 0xA5, float latents and metadata NaN
        self.poison = poison
        fill = (0xFF if latent_dtype in ("f32", "bf16") else 0xA5) if poison else 0
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
    def upload(self, oc: O.LatentCache, n_rows=None, keep_poison=True):
        """Rows [0, n_rows) of the oracle's cache -> device (default: up to the longest sequence).  With keep_poison
        the rows at and past each sequence's length are NOT the oracle's clean zeros but the poison pattern of the
        constructor (codes 0xA5, metadata fp16 NaN, float latents NaN), so that the device planes look like memory the
        append never wrote: a kernel that lets such a row reach a result fails its parity test."""
        lens = oc.seq_lens.astype(np.int64)
        n_rows = int(n_rows or lens.max())
        if n_rows > 0:
            past = np.arange(n_rows)[None, None, :] >= lens[:, None, None]          # [B, 1, n_rows]
            past = np.broadcast_to(past, (oc.k.shape[0], oc.k.shape[1], n_rows))
            for plane, codes, scale, zero in ((0, oc.k, oc.k_scale, oc.k_zero), (1, oc.v, oc.v_scale, oc.v_zero)):
                host = np.ascontiguousarray(codes[:, :, :n_rows]).copy()
                if keep_poison and self.poison:
                    raw = host.view(np.uint8).reshape(host.shape[0], host.shape[1], n_rows, -1)
                    raw[past] = 0xFF if oc.dtype in ("f32", "bf16") else 0xA5
                lc = dev(host)
                meta = None
                if oc.dtype == "i8":
                    m = scale[:, :, :n_rows].view(np.uint16).copy()
                    if keep_poison and self.poison:
                        m[past] = 0xFFFF
                    meta = dev(m)
                elif oc.dtype == "i4":
                    m = np.stack([scale[:, :, :n_rows].view(np.uint16), zero[:, :, :n_rows].view(np.uint16)], axis=-1).copy()
                    if keep_poison and self.poison:
                        m[past] = 0xFFFF
                    meta = dev(m)
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


def check_i8_rows(got_codes, got_scale, values64, what, code_tol=1e-3, scale_tol=1e-5):
    """Symmetric int8 rows written by the GPU from fp32 values that may differ from the oracle's fp64 ones in the last
    bits, against the oracle's quantiser applied to those fp64 values.  values64 [N, r] are the oracle's values before
    quantisation, got_codes [N, r] int8, got_scale [N] fp16.  Accepted, and counted in the return value:
      * a code one step away from the oracle's, only where value / scale lies within code_tol of a .5 rounding boundary;
      * a scale one fp16 step away from the oracle's, only where max|row| / 127 lies within scale_tol (relative) of the
        midpoint between the two fp16 neighbours.  (The fp16 spacing is itself 5e-4 .. 1e-3 relative, so a looser bound
        would accept any row; 1e-5 is about 2 % of the spacing and covers what an fp32 evaluation of the maximum can
        move.)  The codes of such a row are still checked, against the rule applied with the GPU's scale.
    Anything else fails."""
    v = np.asarray(values64, np.float64)
    v = v.reshape(-1, v.shape[-1])
    g = np.asarray(got_codes).reshape(v.shape).astype(np.int64)
    gs = np.asarray(got_scale).reshape(-1).view(np.float16)
    ref_codes, ref_scale = O.quantize_int8_rows(v.astype(np.float32))
    r = ref_codes.astype(np.int64)
    gbits = gs.view(np.uint16).astype(np.int64); rbits = ref_scale.view(np.uint16).astype(np.int64)
    same = gbits == rbits
    flips = 0
    # rows whose scale agrees: codes equal, or one step apart on a rounding boundary
    s64 = ref_scale.astype(np.float64)[:, None]
    bad = (g != r) & same[:, None]
    if bad.any():
        assert np.abs(g - r)[bad].max() == 1, f"{what}: a code is off by more than one step"
        x = (v / s64)[bad]
        frac = np.abs(x - np.floor(x) - 0.5)
        assert frac.max() < code_tol, f"{what}: code differs away from a rounding boundary (distance {frac.max():.3e} steps)"
        flips += int(bad.sum())
    # rows whose scale differs: neighbours in fp16, the exact scale on their midpoint, codes right under the GPU's scale
    for i in np.nonzero(~same)[0]:
        assert abs(int(gbits[i]) - int(rbits[i])) == 1, f"{what}: row {i}: scales {gs[i]} / {ref_scale[i]} are not fp16 neighbours"
        a127 = np.abs(v[i]).max() / 127.0
        mid = 0.5 * (float(gs[i]) + float(ref_scale[i]))
        assert abs(a127 - mid) <= scale_tol * mid, \
            f"{what}: row {i}: scale differs away from an fp16 rounding boundary (max/127 = {a127!r}, boundary {mid!r})"
        x = v[i] / float(gs[i])
        e = np.clip(np.rint(x), -127, 127).astype(np.int64)
        d = g[i] != e
        if d.any():
            assert np.abs(g[i] - e)[d].max() == 1, f"{what}: row {i}: a code is off by more than one step"
            frac = np.abs(x[d] - np.floor(x[d]) - 0.5)
            assert frac.max() < code_tol, f"{what}: row {i}: code differs away from a rounding boundary"
            flips += int(d.sum())
        flips += 1
    return flips
