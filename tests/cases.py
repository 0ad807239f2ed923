"""Build a workload as the oracle sees it (numpy, logical formats) from the seeded generator.
Used by the GPU parity tests, the smoke test and the benchmark's CPU-baseline leg."""
from __future__ import annotations

import numpy as np

import oracle as O
import wsvd_inputs as WI


def round_up(x, m):
    return (x + m - 1) // m * m


class Case:
    pass


def build_case(name, layer=0, extra_cap=64, **over) -> Case:
    """Returns an object with: sp, AK/AV/BK/BV (fp32), lens, cache (oracle LatentCache, filled to lens),
    q32 [B,Hq,d] fp32 query of the next token, x_new [B,E] fp32 hidden state of the next token, sm_scale."""
    sp = WI.spec(name, **over)
    c = Case()
    c.sp = sp
    c.AK, c.AV, c.BK, c.BV = WI.factors(sp, layer)
    c.lens = WI.ragged_lengths(sp)
    c.t_cap = round_up(int(c.lens.max()) + sp.steps + extra_cap, 64)
    c.sm_scale = float(np.float32(1.0 / np.sqrt(sp.d_head)))
    cache = O.LatentCache(sp.batch, sp.n_kv_heads, c.t_cap, sp.rank, sp.latent_dtype)
    if sp.latent_dtype in ("f32", "bf16"):
        # context rows are real projections of hidden states (image-token prefix at image_sigma)
        AK64, AV64 = c.AK.astype(np.float64), c.AV.astype(np.float64)
        for b in range(sp.batch):
            n = int(c.lens[b])
            X = WI.hidden_states(sp, n, 1.0, which="ctx", sub=b).astype(np.float64)
            X[: min(sp.image_tokens, n)] *= sp.image_sigma
            if sp.factor_dtype == "bf16":
                X = WI.bf16_exact(X.astype(np.float32)).astype(np.float64)
            cache.store_rows("k", b, 0, np.transpose(O.project_latents(X, AK64), (1, 0, 2)))
            cache.store_rows("v", b, 0, np.transpose(O.project_latents(X, AV64), (1, 0, 2)))
            cache.seq_lens[b] = n
    else:
        for b in range(sp.batch):
            n = int(c.lens[b])
            cache.store_rows("k", b, 0, WI.latents_from_law(sp, c.AK, "k", b, n, layer).astype(np.float64))
            cache.store_rows("v", b, 0, WI.latents_from_law(sp, c.AV, "v", b, n, layer).astype(np.float64))
            cache.seq_lens[b] = n
    c.cache = cache
    c.x_new = WI.hidden_states(sp, sp.batch * sp.steps, 1.0, which="new").reshape(sp.steps, sp.batch, sp.d_model)
    WQ = WI.dense_wq(sp)
    c.q32 = (c.x_new.astype(np.float64) @ WQ.astype(np.float64)).astype(np.float32).reshape(sp.steps, sp.batch, sp.n_q_heads, sp.d_head)
    return c


def build_block_case(name, layer=0, **over) -> Case:
    """build_case plus the int4 weights of the quantised attention block: W_Q [Hq*d, E], A_K / A_V [Hkv*r, E]
    (output channel kv*r + j) and W_O [E, Hq*d], each as (codes int8 in [-8,7], fp16 scale per output channel),
    and the int8 activation of the next token as the oracle's quantiser leaves it."""
    import dataclasses
    c = build_case(name, layer=layer, **over)
    sp = c.sp
    c.wq = WI.int4_weight(sp, sp.n_q_heads * sp.d_head, 0, layer)
    c.ak = WI.int4_weight(sp, sp.n_kv_heads * sp.rank, 1, layer)
    c.av = WI.int4_weight(sp, sp.n_kv_heads * sp.rank, 2, layer)
    c.wo = WI.int4_weight(dataclasses.replace(sp, d_model=sp.n_q_heads * sp.d_head), sp.d_model, 3, layer)
    c.x32 = c.x_new[0].astype(np.float32)
    c.x_codes, c.x_scale = O.quantize_act_i8(c.x32)
    return c
