"""fp64 / exact-integer oracle of the WSVD decode step (TEST INFRASTRUCTURE ONLY).

What is computed, and where the paper defines it
------------------------------------------------
* latent projection of a token, ``c_Kh = x A_Kh`` and ``c_Vh = x A_Vh``
  (Section 3.1, the per-head decomposition W_Kh = A_Kh B_Kh and the latent
  C_Kh = X A_Kh; Section 3.4 decoding pipeline: the new token is down-projected
  and its K and V latents are stored in the cache);
* storage of the latent row: fp32, bf16, or quantised.  The paper fixes only
  "per-token symmetric" activation quantisation (Section 4.2); the exact rounding
  rules used here are this build's reading and are written out in
  ``quantize_int8_rows`` / ``quantize_int4_rows``;
* attention: K_h = C_Kh B_Kh and V_h = C_Vh B_Vh are MATERIALISED (the "naive
  reconstruction" schedule of Section 3.4, Fig. 4(a)), then plain max-subtracted
  softmax attention of the single query against them;
* a second routine computes the same result with B_K folded into the query and B_V
  applied after the weighted sum of value latents (the algebraic regrouping behind the
  fused kernel of Section 3.4); it exists only to cross-check the first;
* the closed forms of Eq. 2 and Eq. 3 (traffic ratio r/R, parameter ratio rho_1,
  cache ratio rho_2);
* for the full attention block: per-token symmetric int8 activation quantisation and an
  int4-weight x int8-activation linear layer with exact integer accumulation
  (Section 4.2: weights round-to-nearest per-channel symmetric, activations per-token
  symmetric).

* the rest of the decoding pipeline of Section 3.4 (decoding-pipeline figure): the query is per-head low-rank
  too, ``c_Qh = x A_Qh`` up-projected to ``q_h = c_Qh B_Qh``, and the V-path up-projection ``B_Vh`` is fused into
  the output projection; ``fold_qk`` / ``fold_vo`` are those two offline products and ``decode_attn_latent_out`` the
  regrouped attention that consumes them (pinned to the plain definition by associativity); ``decoder_layer_w4a8``
  strings a whole pre-norm decoder layer together in the quantised setting of Section 4.2.

Parity pins (tests/test_oracle_pins.py): identity factors reduce to library attention;
absorbed == reconstructed; softmax rows sum to one; single-row cache returns that V row;
zero query returns the mean V row; a two-token scalar case by hand; row-permutation
invariance; large-score stability; quantiser round trip within one step; nibble packing
exhaustive; one-hot token reproduces a row of A; the printed instance of Eq. 3
(rho_2 = 50 % gives rho_1 ~ 51.5 %, Section 4.4) and the 25 % cache figure of Section 4.2.
The pipeline functions: low-rank-Q attention and the latent-space output against torch attention on tensors formed by
einsum, the folds by associativity, RMSNorm / SiLU against torch, the int4 weight quantiser by invariants and a hand
case, the layer's glue re-done with torch ops.
The numeric value of the output on Gaussian inputs is not printed anywhere in the paper:
for that, parity rests on the pins above.

Conventions: x [B,E]; A_K, A_V [Hkv,E,r]; B_K, B_V [Hkv,r,d]; q [B,Hq,d];
kv(h) = h // (Hq // Hkv).  bf16 values are carried as uint16 bit patterns, fp16 as
numpy float16.  No blocking, fusion or reordering beyond the definitions.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits_from_f32", "f64_from_bf16_bits", "to_f64",
    "quantize_int8_rows", "dequantize_int8_rows",
    "quantize_int4_rows", "dequantize_int4_rows", "pack_int4", "unpack_int4",
    "LatentCache", "project_latents", "latent_append", "latent_prefill", "causal_attn_reconstructed",
    "dequant_cache_rows", "decode_attn_reconstructed", "decode_attn_absorbed", "decode_attn_shared_latent",
    "rope_inv_freq", "rope_rotate", "decode_attn_rope_reconstructed",
    "softmax_weights",
    "traffic_ratio", "param_ratio_rho1", "cache_ratio_rho2", "cache_row_bytes",
    "latent_cache_bytes",
    "quantize_act_i8", "pack_w4", "unpack_w4", "linear_w4a8", "linear_w4a8_int_accum",
    "attention_block_w4a8",
    "up_project_q", "fold_qk", "fold_vo", "decode_attn_lowrank_q", "decode_attn_latent_out",
    "quantize_w4_rows", "rmsnorm", "silu", "decoder_layer_w4a8",
]

# --------------------------------------------------------------------------- storage formats


def bf16_bits_from_f32(x32: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even on the dropped 16 bits); returns uint16 bits.

    NaN is not expected in this workload; infinities pass through unchanged.
    """
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    rounded = (u + 0x7FFF + lsb) >> 16
    return rounded.astype(np.uint16).reshape(x32.shape)


def f64_from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    u = bits.astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64).reshape(bits.shape)


def to_f64(arr: np.ndarray, dtype: str) -> np.ndarray:
    """Exact conversion of a stored tensor ("f32", "bf16", "f16") to fp64."""
    if dtype == "f32":
        return np.asarray(arr, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return f64_from_bf16_bits(arr)
    if dtype == "f16":
        return np.asarray(arr, dtype=np.float16).astype(np.float64)
    raise ValueError(f"to_f64: unsupported dtype {dtype}")


# --------------------------------------------------------------------------- quantisers
# The paper states the granularity (per-token symmetric, Section 4.2) and nothing else.
# The rules below are this build's normative reading; all arithmetic is IEEE fp32 with
# round-to-nearest-even and true division, so that a GPU can reproduce it bit for bit.

_F16_TINY = np.float16(2.0 ** -24)   # smallest positive fp16 (subnormal)
_F16_MAX = np.float16(65504.0)


def _guard_scale_f16(s32: np.ndarray) -> np.ndarray:
    """fp32 scale -> fp16 (RNE) with the zero / overflow guards."""
    with np.errstate(over="ignore"):
        s16 = s32.astype(np.float16)
    s16 = np.where(s16 == 0, _F16_TINY, s16)
    s16 = np.where(np.isinf(s16), _F16_MAX, s16)
    return s16.astype(np.float16)


def quantize_int8_rows(c32: np.ndarray):
    """Symmetric int8, one fp16 scale per row (= per token per head).

    a = max|c_j|; a == 0 -> scale 1, codes 0.  Otherwise s = fp16(a / 127) (guarded),
    code_j = clamp(rint(c_j / float(s)), -127, 127).  Returns (codes int8 [...,r],
    scale fp16 [...]).
    """
    c32 = np.asarray(c32, dtype=np.float32)
    a = np.max(np.abs(c32), axis=-1)
    s32 = a / np.float32(127.0)
    s16 = _guard_scale_f16(s32)
    s16 = np.where(a == 0, np.float16(1.0), s16).astype(np.float16)
    sf = s16.astype(np.float32)[..., None]
    codes = np.clip(np.rint(c32 / sf), -127, 127).astype(np.int8)
    return codes, s16


def dequantize_int8_rows(codes: np.ndarray, scale16: np.ndarray) -> np.ndarray:
    """fp64 value of the stored row: code * scale (exact)."""
    return codes.astype(np.float64) * np.asarray(scale16, dtype=np.float16).astype(np.float64)[..., None]


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """Codes in [0,15], last dim even -> bytes; element 2i in the LOW nibble of byte i."""
    codes = np.asarray(codes).astype(np.uint8)
    assert codes.shape[-1] % 2 == 0
    lo = codes[..., 0::2]
    hi = codes[..., 1::2]
    return (lo | (hi << 4)).astype(np.uint8)


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    packed = np.asarray(packed, dtype=np.uint8)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = packed & 0x0F
    out[..., 1::2] = packed >> 4
    return out


def quantize_int4_rows(c32: np.ndarray):
    """Asymmetric int4, one group per row, fp16 scale and integer-valued fp16 zero point.

    lo = min(min_j c_j, 0), hi = max(max_j c_j, 0); hi == lo -> s=1, z=0, codes 0.
    s = fp16((hi - lo) / 15) (guarded); z = clamp(rint(-lo / float(s)), 0, 15);
    code_j = clamp(int(rint(c_j / float(s))) + int(z), 0, 15).
    Returns (packed uint8 [...,r/2], scale fp16 [...], zero fp16 [...]).
    """
    c32 = np.asarray(c32, dtype=np.float32)
    lo = np.minimum(np.min(c32, axis=-1), np.float32(0))
    hi = np.maximum(np.max(c32, axis=-1), np.float32(0))
    flat = hi == lo
    s32 = (hi - lo) / np.float32(15.0)
    s16 = _guard_scale_f16(s32)
    s16 = np.where(flat, np.float16(1.0), s16).astype(np.float16)
    sf = s16.astype(np.float32)
    z = np.abs(np.clip(np.rint(-lo / sf), 0, 15))     # an integer in [0,15]: lo == 0 must give +0, not -0
    z = np.where(flat, np.float32(0), z).astype(np.float32)
    code = np.rint(c32 / sf[..., None]).astype(np.int64) + z.astype(np.int64)[..., None]
    code = np.clip(code, 0, 15).astype(np.uint8)
    return pack_int4(code), s16, z.astype(np.float16)


def dequantize_int4_rows(packed: np.ndarray, scale16: np.ndarray, zero16: np.ndarray) -> np.ndarray:
    code = unpack_int4(packed).astype(np.float64)
    z = np.asarray(zero16, dtype=np.float16).astype(np.float64)[..., None]
    s = np.asarray(scale16, dtype=np.float16).astype(np.float64)[..., None]
    return (code - z) * s


# --------------------------------------------------------------------------- the latent cache


class LatentCache:
    """Logical per-head latent cache (Section 3.1): row t of head h of sequence b.

    latent_dtype "f32": k/v float32 [B,Hkv,t_cap,r]
                 "bf16": uint16 bit patterns [B,Hkv,t_cap,r]
                 "i8":   int8 codes [B,Hkv,t_cap,r] + fp16 scale [B,Hkv,t_cap]
                 "i4":   packed uint8 [B,Hkv,t_cap,r/2] + fp16 scale, fp16 zero point
    seq_lens int32 [B] = number of valid rows.
    """

    def __init__(self, batch, n_kv_heads, t_cap, rank, latent_dtype):
        self.B, self.Hkv, self.t_cap, self.r, self.dtype = batch, n_kv_heads, t_cap, rank, latent_dtype
        shp = (batch, n_kv_heads, t_cap)
        if latent_dtype == "f32":
            self.k = np.zeros(shp + (rank,), np.float32); self.v = np.zeros(shp + (rank,), np.float32)
        elif latent_dtype == "bf16":
            self.k = np.zeros(shp + (rank,), np.uint16); self.v = np.zeros(shp + (rank,), np.uint16)
        elif latent_dtype == "i8":
            self.k = np.zeros(shp + (rank,), np.int8); self.v = np.zeros(shp + (rank,), np.int8)
        elif latent_dtype == "i4":
            self.k = np.zeros(shp + (rank // 2,), np.uint8); self.v = np.zeros(shp + (rank // 2,), np.uint8)
        else:
            raise ValueError(latent_dtype)
        quant = latent_dtype in ("i8", "i4")
        self.k_scale = np.ones(shp, np.float16) if quant else None
        self.v_scale = np.ones(shp, np.float16) if quant else None
        self.k_zero = np.zeros(shp, np.float16) if latent_dtype == "i4" else None
        self.v_zero = np.zeros(shp, np.float16) if latent_dtype == "i4" else None
        self.seq_lens = np.zeros(batch, np.int32)

    def store_rows(self, which, b, t0, c64):
        """Round fp64 latents c64 [Hkv,n,r] to the storage format and write rows t0..t0+n of sequence b."""
        n = c64.shape[1]
        c32 = c64.astype(np.float32)
        codes = self.k if which == "k" else self.v
        scale = self.k_scale if which == "k" else self.v_scale
        zero = self.k_zero if which == "k" else self.v_zero
        if self.dtype == "f32":
            codes[b, :, t0:t0 + n] = c32
        elif self.dtype == "bf16":
            codes[b, :, t0:t0 + n] = bf16_bits_from_f32(c32)
        elif self.dtype == "i8":
            cq, s = quantize_int8_rows(c32)
            codes[b, :, t0:t0 + n] = cq; scale[b, :, t0:t0 + n] = s
        else:
            cq, s, z = quantize_int4_rows(c32)
            codes[b, :, t0:t0 + n] = cq; scale[b, :, t0:t0 + n] = s; zero[b, :, t0:t0 + n] = z


def project_latents(x64: np.ndarray, A64: np.ndarray) -> np.ndarray:
    """c[b,h,:] = sum_e x[b,e] A[h,e,:]  (C_Kh = X A_Kh, Section 3.1).  x [B,E], A [Hkv,E,r] -> [B,Hkv,r]."""
    B, E = x64.shape
    Hkv, E2, r = A64.shape
    assert E == E2
    out = np.empty((B, Hkv, r), np.float64)
    for h in range(Hkv):
        out[:, h, :] = x64 @ A64[h]
    return out


def latent_append(cache: LatentCache, x64: np.ndarray, AK64: np.ndarray, AV64: np.ndarray):
    """Decode-step cache update (Section 3.4): project the new token of every sequence and
    store its K and V latents at row seq_lens[b]; seq_lens[b] += 1.  A sequence already at
    capacity is left untouched; the returned bool array flags those."""
    cK = project_latents(x64, AK64)
    cV = project_latents(x64, AV64)
    overflow = np.zeros(cache.B, bool)
    for b in range(cache.B):
        n = int(cache.seq_lens[b])
        if n >= cache.t_cap:
            overflow[b] = True
            continue
        cache.store_rows("k", b, n, cK[b][:, None, :])
        cache.store_rows("v", b, n, cV[b][:, None, :])
        cache.seq_lens[b] = n + 1
    return overflow


def latent_prefill(cache: LatentCache, b: int, X64: np.ndarray, AK64: np.ndarray, AV64: np.ndarray) -> bool:
    """Prefill of one sequence (Section 3.4: the input sequence is projected into low-rank latents and the K, V latents
    are stored as the cache): X [n,E] are consecutive tokens of sequence b; token i goes to row seq_lens[b] + i.
    Rows beyond t_cap are dropped and the sequence is left full; returns True in that case."""
    n0 = int(cache.seq_lens[b])
    n_fit = max(0, min(X64.shape[0], cache.t_cap - n0))
    if n_fit:
        cache.store_rows("k", b, n0, np.transpose(project_latents(X64[:n_fit], AK64), (1, 0, 2)))
        cache.store_rows("v", b, n0, np.transpose(project_latents(X64[:n_fit], AV64), (1, 0, 2)))
    cache.seq_lens[b] = n0 + n_fit
    return n_fit < X64.shape[0]


def dequant_cache_rows(cache: LatentCache, which: str, b: int, kv: int, n: int) -> np.ndarray:
    """fp64 value of the first n stored rows of one (sequence, kv head): [n, r]."""
    codes = (cache.k if which == "k" else cache.v)[b, kv, :n]
    if cache.dtype == "f32":
        return codes.astype(np.float64)
    if cache.dtype == "bf16":
        return f64_from_bf16_bits(codes)
    scale = (cache.k_scale if which == "k" else cache.v_scale)[b, kv, :n]
    if cache.dtype == "i8":
        return dequantize_int8_rows(codes, scale)
    zero = (cache.k_zero if which == "k" else cache.v_zero)[b, kv, :n]
    return dequantize_int4_rows(codes, scale, zero)


# --------------------------------------------------------------------------- attention


def softmax_weights(s: np.ndarray) -> np.ndarray:
    """Max-subtracted softmax of a score vector in fp64."""
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


def _heads(q64, BK64):
    B, Hq, d = q64.shape
    Hkv = BK64.shape[0]
    assert Hq % Hkv == 0
    return B, Hq, d, Hkv, Hq // Hkv


def decode_attn_reconstructed(cache: LatentCache, q64: np.ndarray, BK64: np.ndarray, BV64: np.ndarray,
                              sm_scale: float, heads=None) -> np.ndarray:
    """The definition: K = C_K B_K and V = C_V B_V materialised per head (Section 3.1 and the
    naive schedule of Section 3.4), then o = softmax(sm_scale * q K^T) V.

    q64 [B,Hq,d] fp64 (already dequantised), BK64/BV64 [Hkv,r,d].  Returns [B,Hq,d] fp64.
    A sequence with no rows yields zeros.  ``heads`` optionally restricts the (b,h) pairs
    computed (others are left as NaN) so that sampled outputs of a large case stay cheap.
    """
    B, Hq, d, Hkv, G = _heads(q64, BK64)
    out = np.full((B, Hq, d), np.nan) if heads is not None else np.zeros((B, Hq, d))
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(Hq)]
    for (b, h) in pairs:
        n = int(cache.seq_lens[b]); kv = h // G
        if n == 0:
            out[b, h] = 0.0
            continue
        K = dequant_cache_rows(cache, "k", b, kv, n) @ BK64[kv]      # [n,d]
        V = dequant_cache_rows(cache, "v", b, kv, n) @ BV64[kv]      # [n,d]
        s = sm_scale * (K @ q64[b, h])                               # [n]
        p = softmax_weights(s)
        out[b, h] = p @ V
    return out


def decode_attn_shared_latent(cache: LatentCache, q64: np.ndarray, BK64: np.ndarray, BV64: np.ndarray,
                              sm_scale: float, heads=None) -> np.ndarray:
    """The conventional whole-matrix scheme the method is contrasted with (Section 3.1, its figure's panel (b), and the
    "W/o per-head" variant of the latency appendix): ONE latent C_K = X A_K of rank R per token, shared by all heads;
    head h reconstructs K_h = C_K B_Kh with its own B_Kh [R, d] (likewise V_h = C_V B_Vh) and attends as usual:
    o_h = softmax(sm_scale * q_h K_h^T) V_h.

    cache: a LatentCache with ONE kv head of rank R.  q64 [B,H,d], BK64/BV64 [H,R,d].  Returns [B,H,d] fp64; a
    sequence with no rows yields zeros; ``heads`` restricts the (b,h) pairs computed (others NaN)."""
    B, H, d = q64.shape
    assert cache.Hkv == 1 and BK64.shape == (H, cache.r, d) and BV64.shape == (H, cache.r, d)
    out = np.full((B, H, d), np.nan) if heads is not None else np.zeros((B, H, d))
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(H)]
    for (b, h) in pairs:
        n = int(cache.seq_lens[b])
        if n == 0:
            out[b, h] = 0.0
            continue
        K = dequant_cache_rows(cache, "k", b, 0, n) @ BK64[h]        # [n,d]: every head reads the whole shared latent
        V = dequant_cache_rows(cache, "v", b, 0, n) @ BV64[h]
        out[b, h] = softmax_weights(sm_scale * (K @ q64[b, h])) @ V
    return out


def causal_attn_reconstructed(cache: LatentCache, q64: np.ndarray, BK64: np.ndarray, BV64: np.ndarray, sm_scale: float,
                              n_after: int = 0, tokens=None) -> np.ndarray:
    """Attention of several consecutive query tokens per sequence over the cache, each token seeing the rows up to and
    including its own (prefill / multi-token decode; Section 3.4 runs the same reconstruction during prefilling).
    q64 [B,Hkv,nq,G,d]: query token i of sequence b sits at row seq_lens[b] - n_after - nq + i of the cache (the nq
    tokens' latents are already stored, followed by n_after later rows) and attends rows [0, that row].
    K = C_K B_K, V = C_V B_V materialised, plain softmax.  Returns [B,Hkv,nq,G,d]; a token whose row index is negative
    gets zeros.  tokens: optional list of (b, kv, i) to compute; every other entry of the result is NaN (large cases
    are checked on a sample)."""
    B, Hkv, nq, G, d = q64.shape
    if tokens is None:
        out = np.zeros_like(q64)
        todo = [(b, kv, i) for b in range(B) for kv in range(Hkv) for i in range(nq)]
    else:
        out = np.full(q64.shape, np.nan)
        todo = list(tokens)
    for b, kv, i in todo:
        out[b, kv, i] = 0.0
        n_vis = int(cache.seq_lens[b]) - n_after - nq + i + 1
        if n_vis <= 0:
            continue
        K = dequant_cache_rows(cache, "k", b, kv, n_vis) @ BK64[kv]
        V = dequant_cache_rows(cache, "v", b, kv, n_vis) @ BV64[kv]
        for g in range(G):
            out[b, kv, i, g] = softmax_weights(sm_scale * (K @ q64[b, kv, i, g])) @ V
    return out


def rope_inv_freq(d_head: int, base: float) -> np.ndarray:
    """Rotary frequencies theta_i = base^(-2i/d), i < d/2 (fp64)."""
    i = np.arange(d_head // 2, dtype=np.float64)
    return np.float64(base) ** (-2.0 * i / d_head)


def rope_rotate(x64: np.ndarray, pos, base: float) -> np.ndarray:
    """Rotary position embedding in the "rotate-half" pairing: dims (i, i + d/2) form a plane that is turned by the
    angle pos * theta_i:  y_i = x_i cos - x_{i+d/2} sin,  y_{i+d/2} = x_{i+d/2} cos + x_i sin.
    x64 [..., d]; pos broadcastable to x64.shape[:-1]."""
    x = np.asarray(x64, np.float64)
    d = x.shape[-1]
    ang = np.asarray(pos, np.float64)[..., None] * rope_inv_freq(d, base)      # [..., d/2]
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., : d // 2], x[..., d // 2:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def decode_attn_rope_reconstructed(cache: LatentCache, q64: np.ndarray, BK64: np.ndarray, BV64: np.ndarray,
                                   sm_scale: float, rope_base: float, heads=None, pos_offset: float = 0.0) -> np.ndarray:
    """The kernel of Section 3.4 taken literally, for a backbone with rotary position embedding: the key tile
    K = C_K B_K is formed, each key is rotated by its position (its row index), the query by the position of the
    newest row (seq_lens[b] - 1), then o = softmax(sm_scale * q_rot K_rot^T) V with V = C_V B_V.
    With a rotation between the reconstruction and the product, B_K can no longer be folded into the query.
    ``pos_offset`` shifts every position by the same amount (the result must not depend on it)."""
    B, Hq, d, Hkv, G = _heads(q64, BK64)
    out = np.full((B, Hq, d), np.nan) if heads is not None else np.zeros((B, Hq, d))
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(Hq)]
    for (b, h) in pairs:
        n = int(cache.seq_lens[b]); kv = h // G
        if n == 0:
            out[b, h] = 0.0
            continue
        K = dequant_cache_rows(cache, "k", b, kv, n) @ BK64[kv]                  # [n,d]
        V = dequant_cache_rows(cache, "v", b, kv, n) @ BV64[kv]
        K_rot = rope_rotate(K, np.arange(n, dtype=np.float64) + pos_offset, rope_base)
        q_rot = rope_rotate(q64[b, h], np.float64(n - 1) + pos_offset, rope_base)
        s = sm_scale * (K_rot @ q_rot)
        out[b, h] = softmax_weights(s) @ V
    return out


def decode_attn_absorbed(cache: LatentCache, q64: np.ndarray, BK64: np.ndarray, BV64: np.ndarray,
                         sm_scale: float, heads=None) -> np.ndarray:
    """Same result by associativity: q~ = B_K q, s = C_K q~, u = p^T C_V, o = u B_V.
    Used only to cross-check decode_attn_reconstructed (and, being ~d/2 times cheaper, to
    extend sampled checks at the largest shapes after agreeing with it on a subset)."""
    B, Hq, d, Hkv, G = _heads(q64, BK64)
    out = np.full((B, Hq, d), np.nan) if heads is not None else np.zeros((B, Hq, d))
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(Hq)]
    for (b, h) in pairs:
        n = int(cache.seq_lens[b]); kv = h // G
        if n == 0:
            out[b, h] = 0.0
            continue
        qt = BK64[kv] @ q64[b, h]                                    # [r]
        s = sm_scale * (dequant_cache_rows(cache, "k", b, kv, n) @ qt)
        p = softmax_weights(s)
        u = p @ dequant_cache_rows(cache, "v", b, kv, n)             # [r]
        out[b, h] = u @ BV64[kv]
    return out


# --------------------------------------------------------------------------- closed forms (Eq. 2, Eq. 3)


def traffic_ratio(r: int, R: int) -> float:
    """Eq. 2: gamma_wsvd / gamma_svd = eta_wsvd / eta_svd = r / R."""
    return r / R


def param_ratio_rho1(E: int, d_head: int, r: int) -> float:
    """Eq. 3: rho_1 = (E + H) r / (E H) with H the head dimension."""
    return (E + d_head) * r / (E * d_head)


def cache_ratio_rho2(d_head: int, r: int) -> float:
    """Eq. 3: rho_2 = r / H."""
    return r / d_head


def cache_row_bytes(rank: int, latent_dtype: str):
    """(code bytes, metadata bytes) of one stored latent row."""
    bits = {"f32": 32, "bf16": 16, "i8": 8, "i4": 4}[latent_dtype]
    meta = {"f32": 0, "bf16": 0, "i8": 2, "i4": 4}[latent_dtype]
    return rank * bits // 8, meta


def latent_cache_bytes(seq_lens, n_kv_heads: int, rank: int, latent_dtype: str) -> int:
    """Bytes of K plus V latent rows (codes and metadata) that one attention call must read."""
    code, meta = cache_row_bytes(rank, latent_dtype)
    return int(np.sum(np.asarray(seq_lens, dtype=np.int64))) * n_kv_heads * 2 * (code + meta)


# --------------------------------------------------------------------------- W4A8 block (Section 4.2 formats)


def quantize_act_i8(x32: np.ndarray):
    """Per-token symmetric int8 of activation rows [M,K]: same rule as quantize_int8_rows."""
    return quantize_int8_rows(x32)


def pack_w4(w_codes: np.ndarray) -> np.ndarray:
    """Signed int4 weight codes in [-8,7], shape [N,K] (one row per output channel, K even)
    -> two's-complement nibbles, element 2i in the low nibble of byte i: uint8 [N,K/2]."""
    w = np.asarray(w_codes).astype(np.int8)
    assert w.min() >= -8 and w.max() <= 7
    return pack_int4((w.astype(np.int16) & 0xF).astype(np.uint8))


def unpack_w4(packed: np.ndarray) -> np.ndarray:
    u = unpack_int4(packed).astype(np.int16)
    return np.where(u >= 8, u - 16, u).astype(np.int8)


def linear_w4a8_int_accum(x_codes: np.ndarray, w_packed: np.ndarray) -> np.ndarray:
    """Exact integer accumulator acc[m,n] = sum_k x[m,k] * w[n,k] (int64)."""
    w = unpack_w4(w_packed).astype(np.int64)        # [N,K]
    return x_codes.astype(np.int64) @ w.T


def linear_w4a8(x_codes, x_scale16, w_packed, w_scale16) -> np.ndarray:
    """y[m,n] = acc[m,n] * s_x[m] * s_w[n] in fp64 (per-token activation scale, per-output-channel weight scale)."""
    acc = linear_w4a8_int_accum(x_codes, w_packed).astype(np.float64)
    sx = np.asarray(x_scale16, np.float16).astype(np.float64)[:, None]
    sw = np.asarray(w_scale16, np.float16).astype(np.float64)[None, :]
    return acc * sx * sw


def attention_block_w4a8(cache: LatentCache, x_codes, x_scale16, wq_packed, wq_scale16,
                         ak_packed, ak_scale16, av_packed, av_scale16,
                         BK64, BV64, wo_packed, wo_scale16, n_q_heads, d_head, sm_scale, heads=None):
    """One grouped-query attention block in the quantised setting of Section 4.2:
    q = W4A8(x, W_Q); K/V latents of the new token = W4A8(x, A_K), W4A8(x, A_V), stored in
    the cache; decode attention over the cache; o quantised per token to int8; y = W4A8(o, W_O).
    ak_packed / av_packed are [Hkv*r, E/2] with output channel index kv*r + j.
    Returns dict with q, cK, cV (fp64), attn (fp64 [B,Hq,d]), o_codes, o_scale, y (fp64)."""
    B = x_codes.shape[0]
    q = linear_w4a8(x_codes, x_scale16, wq_packed, wq_scale16).reshape(B, n_q_heads, d_head)
    cK = linear_w4a8(x_codes, x_scale16, ak_packed, ak_scale16).reshape(B, cache.Hkv, cache.r)
    cV = linear_w4a8(x_codes, x_scale16, av_packed, av_scale16).reshape(B, cache.Hkv, cache.r)
    for b in range(B):
        n = int(cache.seq_lens[b])
        cache.store_rows("k", b, n, cK[b][:, None, :])
        cache.store_rows("v", b, n, cV[b][:, None, :])
        cache.seq_lens[b] = n + 1
    # the query enters attention in the precision it leaves the projection with (fp32)
    q32 = q.astype(np.float32).astype(np.float64)
    attn = decode_attn_reconstructed(cache, q32, BK64, BV64, sm_scale, heads=heads)
    res = {"q": q, "cK": cK, "cV": cV, "attn": attn}
    if heads is None:
        o_codes, o_scale = quantize_act_i8(attn.reshape(B, n_q_heads * d_head).astype(np.float32))
        res["o_codes"], res["o_scale"] = o_codes, o_scale
        res["y"] = linear_w4a8(o_codes, o_scale, wo_packed, wo_scale16)
    return res


# --------------------------------------------------------------------------- rest of the decoding pipeline (Section 3.4)


def up_project_q(cQ64: np.ndarray, BQ64: np.ndarray) -> np.ndarray:
    """q_h = c_Qh B_Qh (the Q latent is up-projected to form q, Section 3.4): cQ [B,Hq,rq], B_Q [Hq,rq,d] -> [B,Hq,d]."""
    return np.einsum("bhj,hjc->bhc", cQ64, BQ64)


def decode_attn_lowrank_q(cache: LatentCache, cQ64, BQ64, BK64, BV64, sm_scale: float, heads=None) -> np.ndarray:
    """Decode attention of the paper's pipeline, in its order: up-project the Q latent, then attend over the
    materialised K = C_K B_K, V = C_V B_V.  Returns o [B,Hq,d]."""
    return decode_attn_reconstructed(cache, up_project_q(cQ64, BQ64), BK64, BV64, sm_scale, heads=heads)


def fold_qk(BQ64: np.ndarray, BK64: np.ndarray) -> np.ndarray:
    """M_h = B_Qh B_K,kv(h)^T [Hq,rq,r]: q_h K^T = c_Qh B_Qh B_K^T C_K^T = (c_Qh M_h) C_K^T, an offline product."""
    Hq, Hkv = BQ64.shape[0], BK64.shape[0]
    G = Hq // Hkv
    return np.stack([BQ64[h] @ BK64[h // G].T for h in range(Hq)])


def fold_vo(BV64: np.ndarray, WO64: np.ndarray, n_q_heads: int) -> np.ndarray:
    """W'_O [E, Hq*r] with W'_O[:, h*r + j] = sum_c B_V,kv(h)[j,c] W_O[:, h*d + c]: the V up-projection fused into the
    output projection (Section 3.4, following Palu), so that y = W_O o = W'_O u with u the latent-space output.
    W_O is [E, Hq*d] (one row per output channel)."""
    Hkv, r, d = BV64.shape
    G = n_q_heads // Hkv
    E = WO64.shape[0]
    out = np.zeros((E, n_q_heads * r))
    for h in range(n_q_heads):
        out[:, h * r:(h + 1) * r] = WO64[:, h * d:(h + 1) * d] @ BV64[h // G].T
    return out


def decode_attn_latent_out(cache: LatentCache, cQ64: np.ndarray, M64: np.ndarray, sm_scale: float, heads=None) -> np.ndarray:
    """The regrouped attention that goes with the two folds: scores sm_scale * C_K (c_Qh M_h)^T, softmax, and the
    weighted sum of VALUE LATENTS u_h = p^T C_Vh [B,Hq,r]; B_V is never applied (it lives in W'_O)."""
    B, Hq, _ = cQ64.shape
    G = Hq // cache.Hkv
    r = cache.r
    out = np.full((B, Hq, r), np.nan) if heads is not None else np.zeros((B, Hq, r))
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(Hq)]
    for (b, h) in pairs:
        n = int(cache.seq_lens[b]); kv = h // G
        if n == 0:
            out[b, h] = 0.0
            continue
        qt = cQ64[b, h] @ M64[h]                                     # [r]
        s = sm_scale * (dequant_cache_rows(cache, "k", b, kv, n) @ qt)
        out[b, h] = softmax_weights(s) @ dequant_cache_rows(cache, "v", b, kv, n)
    return out


def quantize_w4_rows(W64: np.ndarray):
    """Round-to-nearest per-output-channel symmetric int4 (Section 4.2): rows are output channels.
    a = max|w| of the row; a == 0 -> scale 1, codes 0; else s = fp16(a / 7) (guarded), code = clamp(rint(w / float(s)), -7, 7).
    Returns (codes int8 [N,K], scale fp16 [N])."""
    W32 = np.asarray(W64, dtype=np.float32)
    a = np.max(np.abs(W32), axis=-1)
    s16 = _guard_scale_f16(a / np.float32(7.0))
    s16 = np.where(a == 0, np.float16(1.0), s16).astype(np.float16)
    codes = np.clip(np.rint(W32 / s16.astype(np.float32)[:, None]), -7, 7).astype(np.int8)
    return codes, s16


def rmsnorm(x64: np.ndarray, g64: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * g over the last axis (the pre-norm of a LLaMA-type decoder layer)."""
    return x64 / np.sqrt(np.mean(x64 * x64, axis=-1, keepdims=True) + eps) * g64


def silu(x64: np.ndarray) -> np.ndarray:
    return x64 / (1.0 + np.exp(-x64))


def decoder_layer_w4a8(cache: LatentCache, x32: np.ndarray, g1, g2, wqkv_packed, wqkv_scale16, M64,
                       wo_packed, wo_scale16, wgu_packed, wgu_scale16, wd_packed, wd_scale16,
                       n_q_heads: int, rq: int, sm_scale: float, eps: float = 1e-5):
    """One pre-norm decoder layer of the paper's decoding pipeline in the quantised setting of Section 4.2
    (int4 weights per output channel, int8 activations per token, exact integer sums):

      h1 = rmsnorm(x) g1                       -> int8 per token
      [c_Q | c_K | c_V] = W4A8(h1, [A_Q; A_K; A_V])      (channels h*rq + j, then kv*r + j twice)
      c_K, c_V stored as row seq_lens[b] of the cache (the cache's own quantiser), seq_lens += 1
      u = decode_attn_latent_out(cache, c_Q, M)          (c_Q in the fp32 it leaves the projection with)
      x1 = x + W4A8(int8(u), W'_O)                       (W'_O = the folded output projection, [E, Hq*r])
      h2 = rmsnorm(x1) g2                      -> int8 per token
      [gate | up] = W4A8(h2, [W_g; W_u])       a = silu(gate) * up  -> int8 per token
      x2 = x1 + W4A8(a, W_d)

    The residual stream is fp32 (each sum rounded to fp32).  Returns a dict of every stage."""
    B, E = x32.shape
    Hkv, r = cache.Hkv, cache.r
    f32 = lambda a: np.asarray(a, np.float64).astype(np.float32)
    res = {}
    h1 = f32(rmsnorm(x32.astype(np.float64), np.asarray(g1, np.float64), eps))
    res["h1_codes"], res["h1_scale"] = quantize_act_i8(h1)
    z = linear_w4a8(res["h1_codes"], res["h1_scale"], wqkv_packed, wqkv_scale16)
    nq = n_q_heads * rq
    cQ = z[:, :nq].reshape(B, n_q_heads, rq)
    cK = z[:, nq:nq + Hkv * r].reshape(B, Hkv, r)
    cV = z[:, nq + Hkv * r:].reshape(B, Hkv, r)
    res["cQ"], res["cK"], res["cV"] = cQ, cK, cV
    for b in range(B):
        n = int(cache.seq_lens[b])
        cache.store_rows("k", b, n, cK[b][:, None, :])
        cache.store_rows("v", b, n, cV[b][:, None, :])
        cache.seq_lens[b] = n + 1
    u = decode_attn_latent_out(cache, f32(cQ).astype(np.float64), M64, sm_scale)
    res["u"] = u
    res["u_codes"], res["u_scale"] = quantize_act_i8(f32(u.reshape(B, n_q_heads * r)))
    y = linear_w4a8(res["u_codes"], res["u_scale"], wo_packed, wo_scale16)
    x1 = f32(x32.astype(np.float64) + f32(y).astype(np.float64))
    res["y"], res["x1"] = y, x1
    h2 = f32(rmsnorm(x1.astype(np.float64), np.asarray(g2, np.float64), eps))
    res["h2_codes"], res["h2_scale"] = quantize_act_i8(h2)
    gu = linear_w4a8(res["h2_codes"], res["h2_scale"], wgu_packed, wgu_scale16)
    F = gu.shape[1] // 2
    a = silu(f32(gu[:, :F]).astype(np.float64)) * f32(gu[:, F:]).astype(np.float64)
    res["gu"], res["a"] = gu, a
    res["a_codes"], res["a_scale"] = quantize_act_i8(f32(a))
    dn = linear_w4a8(res["a_codes"], res["a_scale"], wd_packed, wd_scale16)
    res["down"] = dn
    res["x2"] = f32(x1.astype(np.float64) + f32(dn).astype(np.float64))
    return res
