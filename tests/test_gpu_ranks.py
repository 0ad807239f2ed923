"""Per-head ranks other than 32 / 64 (the rank sweep of Eq. 2 / Table 7: r/d = 0.9 .. 0.5 at d = 128, i.e. r = 115, 102,
90, 77, 64).  The library runs ranks 96 and 128 natively (int8 latents); any other rank is zero-padded up to the next
supported one: zero columns of A give zero latent channels, which change neither the row's abs-max nor any product, so
the padded problem has exactly the logical one's result.  The oracle always works at the LOGICAL rank."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
import wsvd_inputs as WI
from cases import build_case
from harness import DeviceLayer, as_dtype_dev, check_i8_rows, err_stats, q_to_device

pytestmark = pytest.mark.gpu

SWEEP = [(115, 128), (102, 128), (90, 96), (77, 96), (96, 96), (128, 128), (64, 64)]


def pad_last(a, r_pad):
    out = np.zeros(a.shape[:-1] + (r_pad,), a.dtype)
    out[..., : a.shape[-1]] = a
    return out


def padded_cache(oc, r_pad):
    """The oracle's cache with every row's codes extended by zero channels (the scales are unchanged)."""
    pc = O.LatentCache(oc.B, oc.Hkv, oc.t_cap, r_pad, "i8")
    pc.k[..., : oc.r] = oc.k; pc.v[..., : oc.r] = oc.v
    pc.k_scale[:] = oc.k_scale; pc.v_scale[:] = oc.v_scale
    pc.seq_lens[:] = oc.seq_lens
    return pc


def device_layer(c, r_pad):
    sp = c.sp
    return DeviceLayer(sp.batch, sp.n_q_heads, sp.n_kv_heads, sp.d_head, sp.d_model, r_pad, c.t_cap, "i8", "bf16", "bf16",
                       sp.q_dtype, c.sm_scale)


def pad_B(Bf, r_pad):          # [Hkv, r, d] -> [Hkv, r_pad, d], zero rows
    out = np.zeros((Bf.shape[0], r_pad, Bf.shape[2]), Bf.dtype)
    out[:, : Bf.shape[1]] = Bf
    return out


@pytest.mark.parametrize("r,r_pad", SWEEP)
def test_attention_at_swept_ranks(r, r_pad):
    c = build_case("c3_small", rank=r)                       # ragged tail: 333 rows, 3 sequences x 4 heads
    c.cache.seq_lens[:] = [333, 64, 129]
    L = device_layer(c, r_pad)
    try:
        L.upload(padded_cache(c.cache, r_pad))
        qd, qs, q64 = q_to_device(c.q32[0], c.sp.q_dtype)
        got = L.attend(qd, qs, as_dtype_dev(pad_B(c.BK, r_pad), "bf16"), as_dtype_dev(pad_B(c.BV, r_pad), "bf16"), 333)
        ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
        a, _, l2 = err_stats(got, ref)
        print(f"rank {r} as {r_pad}: max_abs={a:.3e} rel_l2={l2:.3e}", flush=True)
        assert np.isfinite(got).all() and a <= 2e-2 and l2 <= 1e-3
    finally:
        L.close()


@pytest.mark.parametrize("r,r_pad", [(115, 128), (77, 96), (128, 128)])
def test_append_then_attend_at_swept_ranks(r, r_pad):
    c = build_case("c3_small", rank=r)
    L = device_layer(c, r_pad)
    try:
        L.upload(padded_cache(c.cache, r_pad))
        n0 = c.cache.seq_lens.copy()
        x = WI.bf16_exact(c.x_new[0])
        AK64, AV64 = c.AK.astype(np.float64), c.AV.astype(np.float64)
        cK = O.project_latents(x.astype(np.float64), AK64); cV = O.project_latents(x.astype(np.float64), AV64)     # [B, Hkv, r]
        O.latent_append(c.cache, x.astype(np.float64), AK64, AV64)
        st = L.append(as_dtype_dev(x, "bf16"), None, L.pack_A(pad_last(c.AK, r_pad), "bf16"), L.pack_A(pad_last(c.AV, r_pad), "bf16"))
        assert st == 0, W.status_str(st)
        assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
        for plane, vals in ((0, cK), (1, cV)):
            for b in range(c.sp.batch):
                codes, scale, _ = L.download(plane, int(n0[b]), 1)
                assert (codes[b, :, 0, r:] == 0).all(), "padded channels must stay zero"
                check_i8_rows(codes[b, :, 0, :r], scale[b, :, 0], vals[b], f"rank {r} append plane {plane} seq {b}")
        qd, qs, q64 = q_to_device(c.q32[0], c.sp.q_dtype)
        got = L.attend(qd, qs, as_dtype_dev(pad_B(c.BK, r_pad), "bf16"), as_dtype_dev(pad_B(c.BV, r_pad), "bf16"),
                       int(c.cache.seq_lens.max()))
        ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
        a, _, l2 = err_stats(got, ref)
        assert np.isfinite(got).all() and a <= 2e-2 and l2 <= 1e-3, (a, l2)
    finally:
        L.close()


@pytest.mark.parametrize("r,r_pad", [(115, 128), (90, 96)])
def test_attention_at_swept_ranks_full_shape(r, r_pad):
    """The launch the sweep benchmark times (16 sequences x 32 heads x 2048 rows), on sampled (sequence, head) pairs."""
    c = build_case("c3", rank=r)
    L = device_layer(c, r_pad)
    try:
        L.upload(padded_cache(c.cache, r_pad))
        qd, qs, q64 = q_to_device(c.q32[0], c.sp.q_dtype)
        got = L.attend(qd, qs, as_dtype_dev(pad_B(c.BK, r_pad), "bf16"), as_dtype_dev(pad_B(c.BV, r_pad), "bf16"),
                       int(c.cache.seq_lens.max()))
        assert np.isfinite(got).all()
        rng = np.random.default_rng(5)
        heads = sorted(set((int(b), int(h)) for b, h in zip(rng.integers(0, c.sp.batch, 6), rng.integers(0, c.sp.n_q_heads, 6))))
        ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale, heads=heads)
        mask = ~np.isnan(ref)
        a, _, l2 = err_stats(got[mask], ref[mask])
        print(f"full shape, rank {r} as {r_pad}, (sequence, head) pairs {heads}: max_abs={a:.3e} rel_l2={l2:.3e}", flush=True)
        assert a <= 2e-2 and l2 <= 1e-3
    finally:
        L.close()


def test_wide_ranks_refuse_what_they_do_not_cover():
    d = W.layer_desc(2, 8, 4, 128, 512, 96, 128, "i8", "bf16", "bf16", "i8")       # grouped queries
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_cache_bytes(d)
    assert e.value.status == W.E_UNSUPPORTED
    d = W.layer_desc(2, 4, 4, 128, 512, 128, 128, "i4", "bf16", "bf16", "i8")      # int4 latents
    with pytest.raises(W.WsvdError):
        W.wsvd_cache_bytes(d)


def test_heads_of_different_ranks_by_padding():
    """Rank allocation that differs between the heads of one layer (the appendix's per-head rank search): every head is
    padded with zero columns / rows to the layer's widest supported rank.  The oracle runs each head at its OWN rank;
    the library runs the layer at rank 32 (heads of rank 20, 32, 9 and 27) and at rank 128 (heads of rank 115, 77, 128
    and 64), append and attention."""
    for ranks, r_pad in (([20, 32, 9, 27], 32), ([115, 77, 128, 64], 128)):
        c = build_case("c3_small", rank=r_pad)
        sp = c.sp
        assert sp.n_kv_heads == len(ranks)
        for h, r in enumerate(ranks):                         # zero the padding of every head's factors
            c.AK[h, :, r:] = 0; c.AV[h, :, r:] = 0; c.BK[h, r:] = 0; c.BV[h, r:] = 0
        # the oracle side, head by head at the head's own rank: a one-head cache each
        x = WI.bf16_exact(c.x_new[0]).astype(np.float64)
        ctx_rows = {}
        T0 = int(c.cache.seq_lens.max())
        rng = np.random.default_rng(3)
        Xctx = WI.bf16_exact((rng.standard_normal((sp.batch, T0, sp.d_model)) * 0.8).astype(np.float32)).astype(np.float64)
        ref = np.zeros((sp.batch, sp.n_q_heads, sp.d_head))
        qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
        big = O.LatentCache(sp.batch, sp.n_kv_heads, c.t_cap, r_pad, "i8")
        big.seq_lens[:] = c.cache.seq_lens
        for h, r in enumerate(ranks):
            one = O.LatentCache(sp.batch, 1, c.t_cap, r, "i8")
            AKh, AVh = c.AK[h:h + 1, :, :r].astype(np.float64), c.AV[h:h + 1, :, :r].astype(np.float64)
            for b in range(sp.batch):
                n = int(c.cache.seq_lens[b])
                one.store_rows("k", b, 0, np.transpose(O.project_latents(Xctx[b, :n], AKh), (1, 0, 2)))
                one.store_rows("v", b, 0, np.transpose(O.project_latents(Xctx[b, :n], AVh), (1, 0, 2)))
                one.seq_lens[b] = n
            big.k[:, h, :, :r] = one.k[:, 0]; big.v[:, h, :, :r] = one.v[:, 0]
            big.k_scale[:, h] = one.k_scale[:, 0]; big.v_scale[:, h] = one.v_scale[:, 0]
            O.latent_append(one, x, AKh, AVh)
            ref[:, h] = O.decode_attn_reconstructed(one, q64[:, h:h + 1], c.BK[h:h + 1, :r].astype(np.float64),
                                                    c.BV[h:h + 1, :r].astype(np.float64), c.sm_scale)[:, 0]
        L = device_layer(c, r_pad)
        try:
            L.upload(big)
            st = L.append(as_dtype_dev(x.astype(np.float32), "bf16"), None, L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16"))
            assert st == 0, W.status_str(st)
            got = L.attend(qd, qs, as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16"), int(c.cache.seq_lens.max()) + 1)
            a, _, l2 = err_stats(got, ref)
            print(f"heads of ranks {ranks} run as {r_pad}: max_abs={a:.3e} rel_l2={l2:.3e}", flush=True)
            assert np.isfinite(got).all() and a <= 2e-2 and l2 <= 1e-3
        finally:
            L.close()
