"""Pins for the CPU oracle: each checks it against something other than itself (a library
routine, a closed form, a hand-computed tiny case, an invariant, a value the paper prints)."""
import numpy as np
import pytest
import torch

import oracle as O
from conftest import read_golden


def _rand_cache(rng, B, Hkv, n, r, dtype, t_cap=None, scale=1.0):
    t_cap = t_cap or n
    c = O.LatentCache(B, Hkv, t_cap, r, dtype)
    for b in range(B):
        c.store_rows("k", b, 0, rng.standard_normal((Hkv, n, r)) * scale)
        c.store_rows("v", b, 0, rng.standard_normal((Hkv, n, r)) * scale)
        c.seq_lens[b] = n
    return c


# ---- P1: identity factors with r = d reduce to library attention (torch fp64) -------------
@pytest.mark.parametrize("G", [1, 2])
def test_identity_factors_equal_library_attention(G):
    rng = np.random.default_rng(1)
    B, Hkv, n, d = 2, 3, 37, 8
    Hq = Hkv * G
    cache = _rand_cache(rng, B, Hkv, n, d, "f32")
    q = rng.standard_normal((B, Hq, d))
    I = np.broadcast_to(np.eye(d), (Hkv, d, d)).copy()
    sm = 0.31
    got = O.decode_attn_reconstructed(cache, q, I, I, sm)
    K = torch.from_numpy(cache.k[:, :, :n].astype(np.float64)).repeat_interleave(G, dim=1)  # kv(h) = h // G
    V = torch.from_numpy(cache.v[:, :, :n].astype(np.float64)).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[:, :, None, :], K, V, scale=sm)[:, :, 0].numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_general_factors_equal_library_attention_on_reconstructed_kv():
    """K = C B_K, V = C B_V formed with torch, attention by torch: pins the association and head indexing."""
    rng = np.random.default_rng(2)
    B, Hkv, G, n, r, d = 2, 2, 3, 21, 4, 6
    cache = _rand_cache(rng, B, Hkv, n, r, "f32")
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    q = rng.standard_normal((B, Hkv * G, d))
    got = O.decode_attn_reconstructed(cache, q, BK, BV, 0.5)
    CK = torch.from_numpy(cache.k[:, :, :n].astype(np.float64)); CV = torch.from_numpy(cache.v[:, :, :n].astype(np.float64))
    K = torch.einsum("bhtr,hrd->bhtd", CK, torch.from_numpy(BK)).repeat_interleave(G, dim=1)
    V = torch.einsum("bhtr,hrd->bhtd", CV, torch.from_numpy(BV)).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[:, :, None, :], K, V, scale=0.5)[:, :, 0].numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


# ---- P2: absorbed == reconstructed ---------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16", "i8", "i4"])
def test_absorbed_equals_reconstructed(dtype):
    rng = np.random.default_rng(3)
    B, Hkv, G, n, r, d = 2, 2, 2, 50, 32, 16
    cache = _rand_cache(rng, B, Hkv, n, r, dtype, t_cap=64)
    cache.seq_lens[1] = 17
    BK = rng.standard_normal((Hkv, r, d)) / np.sqrt(r); BV = rng.standard_normal((Hkv, r, d)) / np.sqrt(r)
    q = rng.standard_normal((B, Hkv * G, d))
    a = O.decode_attn_reconstructed(cache, q, BK, BV, d ** -0.5)
    b = O.decode_attn_absorbed(cache, q, BK, BV, d ** -0.5)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


# ---- P3: softmax rows sum to one ----------------------------------------------------------
def test_softmax_sums_to_one_and_matches_scipy():
    from scipy.special import softmax
    rng = np.random.default_rng(4)
    s = rng.standard_normal(1000) * 30
    p = O.softmax_weights(s)
    assert abs(p.sum() - 1) < 1e-14 and (p >= 0).all()
    np.testing.assert_allclose(p, softmax(s), rtol=1e-12, atol=0)


# ---- P4: a single cached token returns that token's V -------------------------------------
def test_single_token_returns_its_value():
    rng = np.random.default_rng(5)
    B, Hkv, r, d = 2, 2, 4, 5
    cache = _rand_cache(rng, B, Hkv, 1, r, "f32", t_cap=3)
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    q = rng.standard_normal((B, Hkv, d)) * 7
    got = O.decode_attn_reconstructed(cache, q, BK, BV, 1.0)
    for b in range(B):
        for h in range(Hkv):
            np.testing.assert_allclose(got[b, h], cache.v[b, h, 0].astype(np.float64) @ BV[h], rtol=1e-13)


# ---- P5: zero query gives the mean value row ---------------------------------------------
def test_zero_query_gives_mean_value():
    rng = np.random.default_rng(6)
    B, Hkv, n, r, d = 1, 2, 13, 4, 5
    cache = _rand_cache(rng, B, Hkv, n, r, "f32")
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    got = O.decode_attn_reconstructed(cache, np.zeros((B, Hkv, d)), BK, BV, 1.0)
    for h in range(Hkv):
        V = cache.v[0, h, :n].astype(np.float64) @ BV[h]
        np.testing.assert_allclose(got[0, h], V.mean(axis=0), rtol=1e-12)


# ---- P6: two tokens, r = d = 1, by hand -----------------------------------------------------
def test_two_token_scalar_case_by_hand():
    import math
    cache = O.LatentCache(1, 1, 2, 1, "f32")
    cache.store_rows("k", 0, 0, np.array([[[0.5], [-1.25]]]))
    cache.store_rows("v", 0, 0, np.array([[[2.0], [3.0]]]))
    cache.seq_lens[0] = 2
    bk, bv, q, sm = 1.5, -0.5, 0.75, 2.0
    got = O.decode_attn_reconstructed(cache, np.array([[[q]]]), np.array([[[bk]]]), np.array([[[bv]]]), sm)[0, 0, 0]
    s1 = sm * q * (0.5 * bk); s2 = sm * q * (-1.25 * bk)
    v1 = 2.0 * bv; v2 = 3.0 * bv
    want = (math.exp(s1) * v1 + math.exp(s2) * v2) / (math.exp(s1) + math.exp(s2))
    assert abs(got - want) < 1e-14


# ---- P7: permuting cache rows (K and V together) leaves the output unchanged ---------------
def test_row_permutation_invariance():
    rng = np.random.default_rng(7)
    B, Hkv, n, r, d = 1, 2, 40, 8, 8
    cache = _rand_cache(rng, B, Hkv, n, r, "i8")
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d)); q = rng.standard_normal((B, Hkv, d))
    a = O.decode_attn_reconstructed(cache, q, BK, BV, 0.3)
    perm = rng.permutation(n)
    for name in ("k", "v", "k_scale", "v_scale"):
        arr = getattr(cache, name)
        arr[:, :, :n] = arr[:, :, perm]
    b = O.decode_attn_reconstructed(cache, q, BK, BV, 0.3)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


# ---- P8: huge scores stay finite and select the arg-max row ---------------------------------
def test_large_scores_select_argmax():
    rng = np.random.default_rng(8)
    B, Hkv, n, r, d = 1, 1, 30, 4, 4
    cache = _rand_cache(rng, B, Hkv, n, r, "f32")
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d)); q = rng.standard_normal((B, Hkv, d))
    got = O.decode_attn_reconstructed(cache, q, BK, BV, 1e4)
    K = cache.k[0, 0, :n].astype(np.float64) @ BK[0]; V = cache.v[0, 0, :n].astype(np.float64) @ BV[0]
    t = int(np.argmax(K @ q[0, 0]))
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got[0, 0], V[t], rtol=1e-9)


# ---- sequence of length zero ---------------------------------------------------------------
def test_empty_sequence_gives_zeros():
    cache = O.LatentCache(2, 1, 4, 2, "f32")
    cache.store_rows("k", 1, 0, np.ones((1, 1, 2))); cache.store_rows("v", 1, 0, np.ones((1, 1, 2))); cache.seq_lens[1] = 1
    out = O.decode_attn_reconstructed(cache, np.ones((2, 1, 3)), np.ones((1, 2, 3)), np.ones((1, 2, 3)), 1.0)
    assert (out[0] == 0).all() and np.allclose(out[1], 2.0)


# ---- P9: quantiser invariants -----------------------------------------------------------------
def test_int8_quantiser_round_trip_and_ranges():
    rng = np.random.default_rng(9)
    c = (rng.standard_normal((500, 32)) * np.exp(rng.standard_normal((500, 1)) * 3)).astype(np.float32)
    c[0] = 0; c[1, 5] = 1e-9; c[2] *= 1e6
    codes, s = O.quantize_int8_rows(c)
    assert codes.dtype == np.int8 and s.dtype == np.float16
    assert codes.min() >= -127 and codes.max() <= 127
    assert (codes[0] == 0).all() and s[0] == np.float16(1.0)
    deq = O.dequantize_int8_rows(codes, s)
    sf = s.astype(np.float64)
    # one-step round trip holds where the fp16 scale is a normal number (relative rounding error <= 2^-11);
    # a saturated scale clamps, and a subnormal scale can under-represent a/127 by more than 1/127
    ok = (sf < 65504) & (sf >= 2.0 ** -14)
    assert ok.sum() > 300
    assert (np.abs(deq - c)[ok] <= sf[ok, None] * 1.0000001 + 0).all()
    # typical rows: the abs-max element lands on +-127
    amax = np.argmax(np.abs(c), axis=1)
    typical = ok & (np.abs(c).max(axis=1) > 1e-3)
    assert (np.abs(codes[np.arange(500), amax])[typical] == 127).all()
    # half-step error away from the clamp
    inner = np.abs(codes) < 127
    assert (np.abs(deq - c)[inner & ok[:, None]] <= 0.5000001 * np.broadcast_to(sf[:, None], c.shape)[inner & ok[:, None]]).all()


def test_int8_quantiser_rounds_half_to_even_and_uses_rounded_scale():
    # a = 127 -> s = 1 exactly; values k + 0.5 must go to the even neighbour
    c = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49]], np.float32)
    codes, s = O.quantize_int8_rows(c)
    assert s[0] == np.float16(1.0)
    assert codes[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 3]
    # a/127 not representable in fp16: the division must use the fp16-rounded scale
    c = np.array([[1000.0, 3.9375, 7.8740234, 500.0]], np.float32)
    codes, s = O.quantize_int8_rows(c)
    s_expect = np.float16(np.float32(1000.0) / np.float32(127.0))
    assert s[0] == s_expect
    assert codes[0].tolist() == [int(np.clip(np.rint(np.float32(v) / np.float32(s_expect)), -127, 127)) for v in c[0]]
    assert codes[0, 0] == 127


def test_int4_quantiser_invariants():
    rng = np.random.default_rng(10)
    c = (rng.standard_normal((400, 32)) * np.exp(rng.standard_normal((400, 1)) * 2) + rng.standard_normal((400, 1))).astype(np.float32)
    c[0] = 0; c[1] = np.abs(c[1]); c[2] = -np.abs(c[2])
    packed, s, z = O.quantize_int4_rows(c)
    assert packed.shape == (400, 16) and packed.dtype == np.uint8
    codes = O.unpack_int4(packed)
    assert codes.max() <= 15
    assert (codes[0] == 0).all() and s[0] == 1 and z[0] == 0
    zf = z.astype(np.float64)
    assert (zf == np.rint(zf)).all() and zf.min() >= 0 and zf.max() <= 15
    assert z[1] == 0                         # all-positive row: range starts at 0
    assert z.view(np.uint16)[1] == 0          # ... stored as +0 (the zero point is an integer code, never -0)
    assert z[2] == 15                        # all-negative row: zero maps to the top code
    deq = O.dequantize_int4_rows(packed, s, z)
    sf = s.astype(np.float64)
    assert (np.abs(deq - c) <= sf[:, None] * 1.0000001).all()
    rows = np.arange(400)
    lo_idx = np.argmin(c, axis=1); hi_idx = np.argmax(c, axis=1)
    has_neg = c.min(axis=1) < 0
    assert (codes[rows, lo_idx][has_neg] <= 1).all()
    has_pos = c.max(axis=1) > 0
    assert (codes[rows, hi_idx][has_pos] >= 14).all()


def test_int4_hand_case():
    # lo = -3, hi = 12 -> s = 1, z = 3; ties to even on c/s
    c = np.array([[-3.0, 12.0, 0.0, 0.5, 1.5, 2.5, -0.5, 7.0]], np.float32)
    packed, s, z = O.quantize_int4_rows(c)
    assert s[0] == 1 and z[0] == 3
    assert O.unpack_int4(packed)[0].tolist() == [0, 15, 3, 3, 5, 5, 3, 10]
    assert packed[0].tolist() == [0 | (15 << 4), 3 | (3 << 4), 5 | (5 << 4), 3 | (10 << 4)]


# ---- P10: nibble packing, exhaustive -------------------------------------------------------
def test_nibble_pack_exhaustive_and_order():
    allb = np.arange(256, dtype=np.uint8)[:, None]
    un = O.unpack_int4(allb)
    assert (un[:, 0] == (allb[:, 0] & 15)).all() and (un[:, 1] == (allb[:, 0] >> 4)).all()
    assert (O.pack_int4(un) == allb).all()
    w = np.arange(-8, 8, dtype=np.int8)[None, :]
    assert (O.unpack_w4(O.pack_w4(w)) == w).all()
    assert O.pack_w4(np.array([[-1, 2]], np.int8))[0, 0] == (0xF | (2 << 4))


def test_bf16_rounding_against_torch():
    rng = np.random.default_rng(11)
    x = (rng.standard_normal(20000) * np.exp(rng.standard_normal(20000) * 5)).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]        # exact ties: to even
    bits = O.bf16_bits_from_f32(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (bits == ref).all()
    back = O.f64_from_bf16_bits(bits)
    assert (back == torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()).all()


# ---- P11: integer GEMM is exact ---------------------------------------------------------------
def test_w4a8_linear_exact_and_scaled():
    rng = np.random.default_rng(12)
    M, K, N = 3, 64, 5
    x = rng.integers(-127, 128, (M, K)).astype(np.int8)
    w = rng.integers(-8, 8, (N, K)).astype(np.int8)
    sx = np.array([0.5, 0.25, 2.0], np.float16); sw = (rng.random(N) + 0.5).astype(np.float16)
    acc = O.linear_w4a8_int_accum(x, O.pack_w4(w))
    brute = np.array([[sum(int(x[m, k]) * int(w[n, k]) for k in range(K)) for n in range(N)] for m in range(M)])
    assert (acc == brute).all()
    y = O.linear_w4a8(x, sx, O.pack_w4(w), sw)
    np.testing.assert_allclose(y, brute * sx.astype(np.float64)[:, None] * sw.astype(np.float64)[None, :], rtol=1e-15)


# ---- P12: closed forms and the values the paper prints -------------------------------------
def test_closed_forms_match_paper_values():
    g = read_golden("paper_printed_values.txt")
    v, tol, _ = g["rho2_at_r64_d128"]
    assert abs(O.cache_ratio_rho2(128, 64) - v) <= tol
    v, tol, _ = g["rho1_at_r64_d128_E4096"]
    assert abs(O.param_ratio_rho1(4096, 128, 64) - v) <= tol
    assert abs(O.param_ratio_rho1(4096, 128, 64) - (1 + 128 / 4096) * 0.5) < 1e-15
    v, tol, _ = g["cache_fraction_int8_rho2_half"]
    code, _meta = O.cache_row_bytes(64, "i8")
    assert abs(code / (128 * 2) - v) <= tol                 # latent codes vs an fp16 K (or V) row of the head
    assert O.traffic_ratio(64, 2048) == 64 / 2048           # Eq. 2
    # byte accounting used for the roofline: config-3 shape
    assert O.latent_cache_bytes([2048] * 16, 32, 32, "i8") == 71303168
    assert O.latent_cache_bytes([257], 8, 16, "f32") == 263168
    assert O.cache_row_bytes(32, "i4") == (16, 4)


# ---- P13: one-hot token reproduces a row of A ---------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_hot_token_appends_row_of_A(dtype):
    rng = np.random.default_rng(13)
    B, Hkv, E, r = 2, 3, 10, 4
    AK = rng.standard_normal((Hkv, E, r)).astype(np.float32); AV = rng.standard_normal((Hkv, E, r)).astype(np.float32)
    cache = O.LatentCache(B, Hkv, 5, r, dtype)
    cache.seq_lens[:] = [2, 0]
    x = np.zeros((B, E)); x[0, 7] = 1.0; x[1, 3] = 1.0
    ov = O.latent_append(cache, x, AK.astype(np.float64), AV.astype(np.float64))
    assert not ov.any() and cache.seq_lens.tolist() == [3, 1]
    for b, e, t in ((0, 7, 2), (1, 3, 0)):
        for h in range(Hkv):
            wantk, wantv = AK[h, e], AV[h, e]
            if dtype == "bf16":
                np.testing.assert_array_equal(cache.k[b, h, t], O.bf16_bits_from_f32(wantk))
                np.testing.assert_array_equal(cache.v[b, h, t], O.bf16_bits_from_f32(wantv))
            else:
                np.testing.assert_array_equal(cache.k[b, h, t], wantk); np.testing.assert_array_equal(cache.v[b, h, t], wantv)
    # untouched rows stay zero; capacity overflow is flagged and leaves the cache alone
    assert (cache.k[0, :, 3:] == 0).all()
    cache.seq_lens[:] = [5, 1]
    before = cache.k.copy()
    ov = O.latent_append(cache, x, AK.astype(np.float64), AV.astype(np.float64))
    assert ov.tolist() == [True, False] and cache.seq_lens.tolist() == [5, 2]
    assert (cache.k[0] == before[0]).all()


def test_projection_matches_einsum():
    rng = np.random.default_rng(14)
    x = rng.standard_normal((3, 11)); A = rng.standard_normal((4, 11, 5))
    np.testing.assert_allclose(O.project_latents(x, A), np.einsum("be,her->bhr", x, A), rtol=1e-13)


def test_append_quantised_matches_quantiser_of_projection():
    rng = np.random.default_rng(15)
    B, Hkv, E, r = 2, 2, 16, 32
    AK = rng.standard_normal((Hkv, E, r)); AV = rng.standard_normal((Hkv, E, r)); x = rng.standard_normal((B, E))
    for dtype in ("i8", "i4"):
        cache = O.LatentCache(B, Hkv, 2, r, dtype)
        O.latent_append(cache, x, AK, AV)
        c32 = np.einsum("be,her->bhr", x, AK).astype(np.float32)
        if dtype == "i8":
            codes, s = O.quantize_int8_rows(c32)
            assert (cache.k[:, :, 0] == codes).all() and (cache.k_scale[:, :, 0] == s).all()
        else:
            codes, s, z = O.quantize_int4_rows(c32)
            assert (cache.k[:, :, 0] == codes).all() and (cache.k_scale[:, :, 0] == s).all() and (cache.k_zero[:, :, 0] == z).all()


def test_attention_block_w4a8_consistency():
    """The block composes the pinned pieces: q and latents are the W4A8 products, y is W4A8 of quantised attention."""
    rng = np.random.default_rng(16)
    B, Hq, Hkv, d, r, E, n = 2, 4, 2, 8, 4, 32, 9
    cache = _rand_cache(rng, B, Hkv, n, r, "i8", t_cap=n + 1)
    xq, xs = O.quantize_act_i8(rng.standard_normal((B, E)).astype(np.float32))
    def w(nout):
        return O.pack_w4(rng.integers(-8, 8, (nout, E)).astype(np.int8)), (rng.random(nout) * 0.1 + 0.05).astype(np.float16)
    wq, wqs = w(Hq * d); ak, aks = w(Hkv * r); av, avs = w(Hkv * r)
    wo = O.pack_w4(rng.integers(-8, 8, (E, Hq * d)).astype(np.int8)); wos = (rng.random(E) * 0.1 + 0.05).astype(np.float16)
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    res = O.attention_block_w4a8(cache, xq, xs, wq, wqs, ak, aks, av, avs, BK, BV, wo, wos, Hq, d, d ** -0.5)
    assert cache.seq_lens.tolist() == [n + 1] * B
    codes, s = O.quantize_int8_rows(res["cK"].astype(np.float32))
    assert (cache.k[:, :, n] == codes).all()
    q32 = res["q"].astype(np.float32).astype(np.float64)
    np.testing.assert_allclose(res["attn"], O.decode_attn_absorbed(cache, q32, BK, BV, d ** -0.5), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(res["y"], O.linear_w4a8(res["o_codes"], res["o_scale"], wo, wos), rtol=0)


def test_attention_block_glue_against_torch():
    """The block's own glue (what lies between the pinned pieces), re-done with torch ops on de-quantised tensors:
    the [B, Hq, d] split of the query projection, the kv*r + j channel split of the two latent projections, the cache
    update, grouped-query attention with K = C B_K, V = C B_V formed by einsum, the [B, Hq*d] flattening that the
    per-token quantiser of o sees, and W_O.  Every head and channel has its own values, and Hq != Hkv, d != r, so a
    transposed reshape, a wrong head / kv mapping or a wrong flattening order changes the result."""
    rng = np.random.default_rng(26)
    B, Hkv, G, n, r, d, E = 3, 2, 3, 21, 8, 16, 32
    Hq = Hkv * G
    cache = _rand_cache(rng, B, Hkv, n, r, "i8", t_cap=n + 2)
    before = (cache.k.copy(), cache.v.copy())
    x32 = (rng.standard_normal((B, E)) * 2).astype(np.float32)
    xq, xs = O.quantize_act_i8(x32)
    def w4(N, K):
        c, s = O.quantize_w4_rows(rng.standard_normal((N, K)) / np.sqrt(K))
        return O.pack_w4(c), s, (c.astype(np.float64) * s.astype(np.float64)[:, None])
    wq_p, wq_s, Wq = w4(Hq * d, E)
    ak_p, ak_s, Ak = w4(Hkv * r, E)
    av_p, av_s, Av = w4(Hkv * r, E)
    wo_p, wo_s, Wo = w4(E, Hq * d)
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    sm = 0.3
    res = O.attention_block_w4a8(cache, xq, xs, wq_p, wq_s, ak_p, ak_s, av_p, av_s, BK, BV, wo_p, wo_s, Hq, d, sm)

    t = torch.from_numpy
    lin = torch.nn.functional.linear
    f32 = lambda a: a.to(torch.float32).to(torch.float64)
    X = t(xq.astype(np.float64) * xs.astype(np.float64)[:, None])          # the de-quantised hidden state
    q = lin(X, t(Wq)); cK = lin(X, t(Ak)); cV = lin(X, t(Av))
    np.testing.assert_allclose(res["q"], q.reshape(B, Hq, d).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(res["cK"], cK.reshape(B, Hkv, r).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(res["cV"], cV.reshape(B, Hkv, r).numpy(), rtol=1e-12, atol=1e-12)
    # cache: old rows untouched, row n = the cache quantiser applied to head kv's slice [kv*r, (kv+1)*r), lengths + 1
    assert (cache.seq_lens == n + 1).all()
    assert (cache.k[:, :, :n] == before[0][:, :, :n]).all() and (cache.v[:, :, :n] == before[1][:, :, :n]).all()
    for kv in range(Hkv):
        kc, ks = O.quantize_int8_rows(cK[:, kv * r:(kv + 1) * r].numpy().astype(np.float32))
        vc, vs = O.quantize_int8_rows(cV[:, kv * r:(kv + 1) * r].numpy().astype(np.float32))
        assert (cache.k[:, kv, n] == kc).all() and (cache.k_scale[:, kv, n] == ks).all()
        assert (cache.v[:, kv, n] == vc).all() and (cache.v_scale[:, kv, n] == vs).all()
    # grouped-query attention over the materialised keys and values; query head h uses kv head h // G
    CK = t(_dequant_all(cache, "k")); CV = t(_dequant_all(cache, "v"))        # [B, Hkv, n + 1, r]
    K = torch.einsum("bktj,kjc->bktc", CK, t(BK)).repeat_interleave(G, dim=1)
    V = torch.einsum("bktj,kjc->bktc", CV, t(BV)).repeat_interleave(G, dim=1)
    qh = f32(q).reshape(B, Hq, 1, d)                                          # fp32 as it leaves the projection
    o = torch.nn.functional.scaled_dot_product_attention(qh, K, V, scale=sm)[:, :, 0]       # [B, Hq, d]
    np.testing.assert_allclose(res["attn"], o.numpy(), rtol=1e-10, atol=1e-11)
    # per-token quantiser over the row [h*d + c], then W_O
    oc, os_ = O.quantize_act_i8(o.reshape(B, Hq * d).numpy().astype(np.float32))
    assert (res["o_codes"] == oc).all() and (res["o_scale"] == os_).all()
    y = lin(t(oc.astype(np.float64) * os_.astype(np.float64)[:, None]), t(Wo))
    np.testing.assert_allclose(res["y"], y.numpy(), rtol=1e-12, atol=1e-12)
    # the pin has teeth: heads differ, so a permuted head order would not pass
    assert np.abs(o[:, 0] - o[:, 1]).max() > 1e-3 and np.abs(o[:, 0] - o[:, G]).max() > 1e-3


# ---- rotary variant (reconstruct, rotate, then q K^T) ---------------------------------------
def test_rope_rotation_is_the_textbook_one():
    """Pairs (i, i + d/2) as complex numbers multiplied by exp(i pos theta_i): an independent formulation."""
    rng = np.random.default_rng(40)
    d, base = 16, 10000.0
    x = rng.standard_normal((5, 7, d)); pos = rng.integers(0, 5000, (5, 7)).astype(np.float64)
    got = O.rope_rotate(x, pos, base)
    theta = np.array([base ** (-2.0 * i / d) for i in range(d // 2)])
    z = (x[..., : d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * pos[..., None] * theta)
    np.testing.assert_allclose(got, np.concatenate([z.real, z.imag], -1), rtol=1e-12, atol=1e-12)
    # d = 2: one plane, a plain 2x2 rotation by the angle pos (theta_0 = 1)
    v = np.array([3.0, -1.5]); a = 0.7
    np.testing.assert_allclose(O.rope_rotate(v, a, 123.0), [v[0] * np.cos(a) - v[1] * np.sin(a), v[1] * np.cos(a) + v[0] * np.sin(a)], atol=1e-15)
    assert np.allclose(O.rope_inv_freq(8, 10000.0), [1.0, 0.1, 0.01, 0.001])


def test_rope_rotation_invariants():
    rng = np.random.default_rng(41)
    d, base = 32, 10000.0
    x = rng.standard_normal((9, d)); y = rng.standard_normal((9, d))
    np.testing.assert_array_equal(O.rope_rotate(x, 0.0, base), x)                                     # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(O.rope_rotate(x, 77.0, base), axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(O.rope_rotate(O.rope_rotate(x, 5.0, base), 11.0, base), O.rope_rotate(x, 16.0, base), atol=1e-12)
    # the product of a rotated query and a rotated key depends on the difference of their positions only
    a = np.sum(O.rope_rotate(x, 100.0, base) * O.rope_rotate(y, 37.0, base), -1)
    b = np.sum(O.rope_rotate(x, 63.0, base) * y, -1)
    c = np.sum(x * O.rope_rotate(y, -63.0, base), -1)
    np.testing.assert_allclose(a, b, atol=1e-11); np.testing.assert_allclose(a, c, atol=1e-11)


@pytest.mark.parametrize("dtype", ["f32", "i8"])
def test_rope_attention_against_torch_and_its_invariants(dtype):
    rng = np.random.default_rng(42)
    B, Hkv, G, n, r, d, base = 2, 2, 3, 37, 8, 16, 10000.0
    cache = _rand_cache(rng, B, Hkv, n, r, dtype)
    cache.seq_lens[1] = 20
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    q = rng.standard_normal((B, Hkv * G, d))
    got = O.decode_attn_rope_reconstructed(cache, q, BK, BV, 0.3, base)
    # K, V formed and rotated with torch / complex arithmetic, attention by torch
    theta = torch.tensor([base ** (-2.0 * i / d) for i in range(d // 2)], dtype=torch.float64)
    def rot(x, pos):
        z = torch.complex(x[..., : d // 2], x[..., d // 2:]) * torch.polar(torch.ones_like(pos[..., None] * theta), pos[..., None] * theta)
        return torch.cat([z.real, z.imag], -1)
    for b in range(B):
        nb = int(cache.seq_lens[b])
        for h in range(Hkv * G):
            kv = h // G
            CK = torch.from_numpy(O.dequant_cache_rows(cache, "k", b, kv, nb)); CV = torch.from_numpy(O.dequant_cache_rows(cache, "v", b, kv, nb))
            K = rot(CK @ torch.from_numpy(BK[kv]), torch.arange(nb, dtype=torch.float64))
            V = CV @ torch.from_numpy(BV[kv])
            qr = rot(torch.from_numpy(q[b, h]), torch.tensor(float(nb - 1), dtype=torch.float64))
            ref = torch.nn.functional.scaled_dot_product_attention(qr[None, None, None, :], K[None, None], V[None, None], scale=0.3)[0, 0, 0].numpy()
            np.testing.assert_allclose(got[b, h], ref, rtol=1e-11, atol=1e-12)
    # shifting every position by the same amount changes nothing
    np.testing.assert_allclose(O.decode_attn_rope_reconstructed(cache, q, BK, BV, 0.3, base, pos_offset=1234.0), got, atol=1e-10)
    # it is NOT the unrotated attention (the rotation matters) ...
    assert np.abs(got - O.decode_attn_reconstructed(cache, q, BK, BV, 0.3)).max() > 1e-3
    # ... except for a single cached token, whose output is its value row whatever the rotation
    one = _rand_cache(rng, 1, Hkv, 1, r, dtype)
    np.testing.assert_allclose(O.decode_attn_rope_reconstructed(one, q[:1], BK, BV, 0.3, base),
                               O.decode_attn_reconstructed(one, q[:1], BK, BV, 0.3), atol=1e-13)
    # the regrouping the GPU kernel uses: s_t = sum_i cos(phi_i) A_i(t) + sin(phi_i) B_i(t), phi_i = theta_i (n-1-t),
    # A_i = q_i k_i + q_i' k_i', B_i = q_i k_i' - q_i' k_i  (i' = i + d/2): checked here against the definition
    b, h, kv = 0, 4, 4 // G
    nb = int(cache.seq_lens[b])
    K = O.dequant_cache_rows(cache, "k", b, kv, nb) @ BK[kv]
    th = O.rope_inv_freq(d, base); half = d // 2
    Ai = q[b, h, :half] * K[:, :half] + q[b, h, half:] * K[:, half:]
    Bi = q[b, h, :half] * K[:, half:] - q[b, h, half:] * K[:, :half]
    phi = (nb - 1 - np.arange(nb))[:, None] * th
    s_regrouped = (np.cos(phi) * Ai + np.sin(phi) * Bi).sum(-1)
    s_def = O.rope_rotate(K, np.arange(nb), base) @ O.rope_rotate(q[b, h], nb - 1, base)
    np.testing.assert_allclose(s_regrouped, s_def, atol=1e-11)


# ---- rest of the decoding pipeline: low-rank Q, B_V folded into W_O, the quantised decoder layer ----------
def _dequant_all(cache, which):
    B, Hkv, n = cache.B, cache.Hkv, int(cache.seq_lens[0])
    return np.stack([np.stack([O.dequant_cache_rows(cache, which, b, kv, n) for kv in range(Hkv)]) for b in range(B)])


@pytest.mark.parametrize("dtype,G", [("f32", 1), ("i8", 2), ("bf16", 3)])
def test_lowrank_q_pipeline_against_torch(dtype, G):
    """q = c_Q B_Q, K = C_K B_K, V = C_V B_V all formed with torch, attention by torch."""
    rng = np.random.default_rng(21)
    B, Hkv, n, r, rq, d = 2, 2, 41, 8, 6, 16
    Hq = Hkv * G
    cache = _rand_cache(rng, B, Hkv, n, r, dtype)
    cQ = rng.standard_normal((B, Hq, rq)); BQ = rng.standard_normal((Hq, rq, d))
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    sm = 0.27
    got = O.decode_attn_lowrank_q(cache, cQ, BQ, BK, BV, sm)
    t = torch.from_numpy
    q = torch.einsum("bhj,hjc->bhc", t(cQ), t(BQ))
    K = torch.einsum("bknr,krc->bknc", t(_dequant_all(cache, "k")), t(BK)).repeat_interleave(G, dim=1)
    V = torch.einsum("bknr,krc->bknc", t(_dequant_all(cache, "v")), t(BV)).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q[:, :, None, :], K, V, scale=sm)[:, :, 0].numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_folds_reproduce_the_unfolded_pipeline():
    """W_O applied to the plain attention output == W'_O applied to the latent-space output of the regrouped
    attention (associativity); the folds themselves against einsum; the latent-space output against torch attention
    whose values are the latent rows."""
    rng = np.random.default_rng(22)
    B, Hkv, G, n, r, rq, d, E = 2, 2, 2, 29, 8, 5, 16, 24
    Hq = Hkv * G
    cache = _rand_cache(rng, B, Hkv, n, r, "i8")
    cQ = rng.standard_normal((B, Hq, rq)); BQ = rng.standard_normal((Hq, rq, d))
    BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    WO = rng.standard_normal((E, Hq * d))
    sm = 0.4
    M = O.fold_qk(BQ, BK); WOf = O.fold_vo(BV, WO, Hq)
    t = torch.from_numpy
    kvmap = torch.arange(Hq) // G
    np.testing.assert_allclose(M, torch.einsum("hjc,hrc->hjr", t(BQ), t(BK)[kvmap]).numpy(), rtol=1e-13, atol=1e-13)
    ref_f = torch.einsum("ehc,hjc->ehj", t(WO).reshape(E, Hq, d), t(BV)[kvmap]).reshape(E, Hq * r).numpy()
    np.testing.assert_allclose(WOf, ref_f, rtol=1e-13, atol=1e-13)
    o = O.decode_attn_lowrank_q(cache, cQ, BQ, BK, BV, sm)
    u = O.decode_attn_latent_out(cache, cQ, M, sm)
    np.testing.assert_allclose(u.reshape(B, Hq * r) @ WOf.T, o.reshape(B, Hq * d) @ WO.T, rtol=1e-10, atol=1e-10)
    # u itself: torch attention with the query c_Q M, keys C_K and VALUES = the latent rows C_V
    qt = torch.einsum("bhj,hjr->bhr", t(cQ), t(M))
    CK = t(_dequant_all(cache, "k")).repeat_interleave(G, dim=1); CV = t(_dequant_all(cache, "v")).repeat_interleave(G, dim=1)
    ref_u = torch.nn.functional.scaled_dot_product_attention(qt[:, :, None, :], CK, CV, scale=sm)[:, :, 0].numpy()
    np.testing.assert_allclose(u, ref_u, rtol=1e-11, atol=1e-12)
    # sampled heads and an empty sequence
    cache.seq_lens[1] = 0
    part = O.decode_attn_latent_out(cache, cQ, M, sm, heads=[(0, 1), (1, 2)])
    np.testing.assert_allclose(part[0, 1], u[0, 1], rtol=0, atol=0)
    assert (part[1, 2] == 0).all() and np.isnan(part[0, 0]).all()


def test_int4_weight_quantiser():
    rng = np.random.default_rng(23)
    W = rng.standard_normal((9, 40)) * np.exp(rng.standard_normal((9, 1)))
    W[3] = 0
    W[4] = 0; W[4, 7] = -3.5                                  # scale fp16(0.5): codes 0 except -7
    codes, s = O.quantize_w4_rows(W)
    assert codes.dtype == np.int8 and s.dtype == np.float16 and codes.min() >= -7 and codes.max() <= 7
    assert (codes[3] == 0).all() and s[3] == 1
    assert s[4] == np.float16(0.5) and codes[4, 7] == -7 and np.count_nonzero(codes[4]) == 1
    sf = s.astype(np.float64)[:, None]
    assert (np.abs(codes * sf - W) <= 0.5 * sf * (1 + 1e-3) + 1e-12).all()          # round to nearest
    for i in range(9):                                       # the largest entry of a row maps to +-7
        if i != 3:
            assert abs(int(codes[i, np.argmax(np.abs(W[i]))])) == 7
    np.testing.assert_array_equal(O.quantize_w4_rows(-W)[0], -codes)           # symmetric
    np.testing.assert_array_equal(O.unpack_w4(O.pack_w4(codes)), codes)


def test_rmsnorm_and_silu_against_torch():
    rng = np.random.default_rng(24)
    x = rng.standard_normal((5, 48)) * 3; g = rng.standard_normal(48)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(O.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-13)
    # unit gain, eps = 0: rows come out with mean square exactly 1
    np.testing.assert_allclose(np.mean(O.rmsnorm(x, np.ones(48), 0.0) ** 2, axis=-1), 1.0, rtol=1e-13)


def test_decoder_layer_glue_against_torch():
    """The layer's order of operations, channel splits, residuals and cache update, re-done with torch linear /
    rms_norm / silu / attention on de-quantised tensors.  The activation and cache quantisers are the oracle's own
    (pinned above); what this pins is everything between them."""
    rng = np.random.default_rng(25)
    B, Hkv, G, n, r, rq, d, E, F = 3, 2, 2, 23, 8, 8, 16, 32, 48
    Hq = Hkv * G
    cache = _rand_cache(rng, B, Hkv, n, r, "i8", t_cap=n + 2)
    before = (cache.k.copy(), cache.v.copy())
    x = (rng.standard_normal((B, E)) * 2).astype(np.float32)
    g1 = 1 + 0.1 * rng.standard_normal(E); g2 = 1 + 0.1 * rng.standard_normal(E)
    def w4(N, K):
        c, s = O.quantize_w4_rows(rng.standard_normal((N, K)) / np.sqrt(K))
        return O.pack_w4(c), s, (c.astype(np.float64) * s.astype(np.float64)[:, None])
    qkv_p, qkv_s, Wqkv = w4(Hq * rq + 2 * Hkv * r, E)
    BQ = rng.standard_normal((Hq, rq, d)); BK = rng.standard_normal((Hkv, r, d))
    M = O.fold_qk(BQ, BK)
    wo_p, wo_s, Wo = w4(E, Hq * r)
    gu_p, gu_s, Wgu = w4(2 * F, E)
    wd_p, wd_s, Wd = w4(E, F)
    sm, eps = 0.25, 1e-5
    res = O.decoder_layer_w4a8(cache, x, g1, g2, qkv_p, qkv_s, M, wo_p, wo_s, gu_p, gu_s, wd_p, wd_s, Hq, rq, sm, eps)

    t = torch.from_numpy
    lin = torch.nn.functional.linear
    fq = lambda a: (lambda c, s: t(c.astype(np.float64) * s.astype(np.float64)[:, None]))(*O.quantize_act_i8(np.asarray(a, np.float32)))
    f32 = lambda a: a.to(torch.float32).to(torch.float64)
    X = t(x.astype(np.float64))
    h1 = fq(f32(torch.nn.functional.rms_norm(X, (E,), t(g1), eps=eps)).numpy())
    z = lin(h1, t(Wqkv))
    cQ = z[:, :Hq * rq].reshape(B, Hq, rq); cK = z[:, Hq * rq:Hq * rq + Hkv * r].reshape(B, Hkv, r); cV = z[:, Hq * rq + Hkv * r:].reshape(B, Hkv, r)
    np.testing.assert_allclose(res["cQ"], cQ.numpy(), rtol=1e-12, atol=1e-12)
    # cache: old rows untouched, row n = the cache quantiser applied to the new latents, lengths advanced
    assert (cache.seq_lens == n + 1).all()
    assert (cache.k[:, :, :n] == before[0][:, :, :n]).all() and (cache.v[:, :, :n] == before[1][:, :, :n]).all()
    kc, ks = O.quantize_int8_rows(cK.numpy().astype(np.float32)); vc, vs = O.quantize_int8_rows(cV.numpy().astype(np.float32))
    assert (cache.k[:, :, n] == kc).all() and (cache.k_scale[:, :, n] == ks).all()
    assert (cache.v[:, :, n] == vc).all() and (cache.v_scale[:, :, n] == vs).all()
    CK = t(_dequant_all(cache, "k")).repeat_interleave(G, dim=1); CV = t(_dequant_all(cache, "v")).repeat_interleave(G, dim=1)
    qt = torch.einsum("bhj,hjr->bhr", f32(cQ), t(M))
    u = torch.nn.functional.scaled_dot_product_attention(qt[:, :, None, :], CK, CV, scale=sm)[:, :, 0]
    np.testing.assert_allclose(res["u"], u.numpy(), rtol=1e-10, atol=1e-11)
    x1 = f32(X + f32(lin(fq(u.reshape(B, Hq * r).numpy()), t(Wo))))
    np.testing.assert_allclose(res["x1"], x1.numpy(), rtol=1e-6, atol=1e-6)
    h2 = fq(f32(torch.nn.functional.rms_norm(x1, (E,), t(g2), eps=eps)).numpy())
    gu = lin(h2, t(Wgu))
    a = torch.nn.functional.silu(f32(gu[:, :F])) * f32(gu[:, F:])
    x2 = f32(x1 + f32(lin(fq(a.numpy()), t(Wd))))
    np.testing.assert_allclose(res["x2"], x2.numpy(), rtol=1e-6, atol=1e-6)
    assert np.abs(res["x2"] - x).max() > 0.1           # the layer does something


def test_prefill_equals_successive_appends():
    """Prefilling n tokens of one sequence == appending them one at a time (the append is pinned above); a prompt that
    does not fit fills the sequence and says so; other sequences are untouched."""
    rng = np.random.default_rng(31)
    Hkv, E, r, n = 2, 24, 8, 11
    AK = rng.standard_normal((Hkv, E, r)); AV = rng.standard_normal((Hkv, E, r))
    X = rng.standard_normal((n, E))
    for dtype in ("f32", "bf16", "i8", "i4"):
        a = _rand_cache(rng, 2, Hkv, 5, r, dtype, t_cap=20)
        b = O.LatentCache(2, Hkv, 20, r, dtype)
        for name in ("k", "v", "k_scale", "v_scale", "k_zero", "v_zero", "seq_lens"):
            if getattr(a, name) is not None:
                getattr(b, name)[...] = getattr(a, name)
        assert O.latent_prefill(a, 1, X, AK, AV) is False
        for i in range(n):                      # one-sequence appends: a batch-1 view would need a second cache type,
            x2 = np.zeros((2, E)); x2[1] = X[i]  # so sequence 0 gets a zero token and is compared up to its old length
            O.latent_append(b, x2, AK, AV)
        assert a.seq_lens.tolist() == [5, 16] and b.seq_lens.tolist() == [16, 16]
        for name in ("k", "v", "k_scale", "v_scale", "k_zero", "v_zero"):
            if getattr(a, name) is not None:
                np.testing.assert_array_equal(getattr(a, name)[1, :, :16], getattr(b, name)[1, :, :16])
                np.testing.assert_array_equal(getattr(a, name)[0, :, :5], getattr(b, name)[0, :, :5])
        assert O.latent_prefill(a, 1, X, AK, AV) is True and a.seq_lens[1] == 20


@pytest.mark.parametrize("dtype,G,n_after", [("f32", 1, 0), ("i8", 2, 3)])
def test_causal_attention_against_torch_mask(dtype, G, n_after):
    """K, V formed with torch, attention by torch with an explicit boolean mask; one query token reduces to the decode
    routine."""
    rng = np.random.default_rng(41)
    B, Hkv, n, r, d, nq = 2, 2, 23, 8, 16, 5
    cache = _rand_cache(rng, B, Hkv, n, r, dtype)
    q = rng.standard_normal((B, Hkv, nq, G, d)); BK = rng.standard_normal((Hkv, r, d)); BV = rng.standard_normal((Hkv, r, d))
    sm = 0.3
    got = O.causal_attn_reconstructed(cache, q, BK, BV, sm, n_after=n_after)
    t = torch.from_numpy
    K = torch.einsum("bknr,krc->bknc", t(_dequant_all(cache, "k")), t(BK))          # [B,Hkv,n,d]
    V = torch.einsum("bknr,krc->bknc", t(_dequant_all(cache, "v")), t(BV))
    pos = n - n_after - nq + torch.arange(nq)                                         # row of query token i
    mask = (torch.arange(n)[None, :] <= pos[:, None])                                 # [nq, n]
    for g in range(G):
        ref = torch.nn.functional.scaled_dot_product_attention(t(q[:, :, :, g]), K, V, attn_mask=mask, scale=sm).numpy()
        np.testing.assert_allclose(got[:, :, :, g], ref, rtol=1e-11, atol=1e-12)
    # a single query token that is the newest row: the decode routine
    q1 = q[:, :, -1:, :, :]
    one = O.causal_attn_reconstructed(cache, q1, BK, BV, sm)
    dec = O.decode_attn_reconstructed(cache, q1.reshape(B, Hkv * G, d), BK, BV, sm)
    np.testing.assert_allclose(one.reshape(B, Hkv * G, d), dec, rtol=1e-12, atol=1e-13)
    # tokens before the start of the sequence get zeros
    cache.seq_lens[:] = 2
    z = O.causal_attn_reconstructed(cache, q, BK, BV, sm)
    assert (z[:, :, :3] == 0).all() and np.abs(z[:, :, 3:]).min() > 0


def test_causal_attention_sample_option_only_selects():
    """The tokens= option of the causal attention computes the same values for the listed (sequence, head, token)
    triples and leaves every other entry NaN."""
    import wsvd_inputs as WI
    from cases import build_case
    c = build_case("c3_small", batch=2, context=40)
    sp = c.sp
    G = sp.n_q_heads // sp.n_kv_heads
    rng = np.random.default_rng(2)
    q = rng.standard_normal((sp.batch, sp.n_kv_heads, 5, G, sp.d_head))
    BK, BV = c.BK.astype(np.float64), c.BV.astype(np.float64)
    full = O.causal_attn_reconstructed(c.cache, q, BK, BV, c.sm_scale, n_after=1)
    toks = [(0, 0, 0), (1, sp.n_kv_heads - 1, 4), (1, 1, 2)]
    part = O.causal_attn_reconstructed(c.cache, q, BK, BV, c.sm_scale, n_after=1, tokens=toks)
    for t in toks:
        assert np.array_equal(part[t], full[t])
    assert np.isnan(part).sum() == part.size - len(toks) * G * sp.d_head


# ------------------------------------------------------------------ shared-latent (whole-matrix) contrast, Section 3.1
def test_shared_latent_attention_brute_force_tiny():
    """Python loops over every index on a tiny case."""
    rng = np.random.default_rng(5)
    B, H, R, d, n = 2, 3, 4, 3, 5
    cache = O.LatentCache(B, 1, 8, R, "f32")
    cache.k[:] = rng.standard_normal(cache.k.shape).astype(np.float32)
    cache.v[:] = rng.standard_normal(cache.v.shape).astype(np.float32)
    cache.seq_lens[:] = [n, 0]
    q = rng.standard_normal((B, H, d)); BK = rng.standard_normal((H, R, d)); BV = rng.standard_normal((H, R, d))
    got = O.decode_attn_shared_latent(cache, q, BK, BV, 0.7)
    assert (got[1] == 0).all()
    for h in range(H):
        s = []
        for t in range(n):
            acc = 0.0
            for c in range(d):
                kc = sum(float(cache.k[0, 0, t, j]) * BK[h, j, c] for j in range(R))
                acc += q[0, h, c] * kc
            s.append(0.7 * acc)
        m = max(s); e = [np.exp(x - m) for x in s]; z = sum(e)
        for c in range(d):
            want = sum(e[t] / z * sum(float(cache.v[0, 0, t, j]) * BV[h, j, c] for j in range(R)) for t in range(n))
            assert abs(got[0, h, c] - want) <= 1e-12 * (1 + abs(want))


def test_shared_latent_with_block_factors_is_the_per_head_scheme():
    """Per-head SVD is the shared scheme with block-structured up-projections: if the shared latent is the heads' latents
    side by side and B_Kh is zero outside head h's block, both schemes give the same attention (fp32 caches, so no
    quantiser in between)."""
    rng = np.random.default_rng(8)
    B, H, r, d, n = 2, 4, 8, 16, 37
    per = O.LatentCache(B, H, 64, r, "f32")
    per.k[:] = rng.standard_normal(per.k.shape).astype(np.float32); per.v[:] = rng.standard_normal(per.v.shape).astype(np.float32)
    per.seq_lens[:] = [n, 11]
    sh = O.LatentCache(B, 1, 64, H * r, "f32")
    sh.k[:, 0] = np.transpose(per.k, (0, 2, 1, 3)).reshape(B, 64, H * r)
    sh.v[:, 0] = np.transpose(per.v, (0, 2, 1, 3)).reshape(B, 64, H * r)
    sh.seq_lens[:] = per.seq_lens
    BK = rng.standard_normal((H, r, d)); BV = rng.standard_normal((H, r, d)); q = rng.standard_normal((B, H, d))
    BKs = np.zeros((H, H * r, d)); BVs = np.zeros((H, H * r, d))
    for h in range(H):
        BKs[h, h * r:(h + 1) * r] = BK[h]; BVs[h, h * r:(h + 1) * r] = BV[h]
    a = O.decode_attn_reconstructed(per, q, BK, BV, 0.3)
    b = O.decode_attn_shared_latent(sh, q, BKs, BVs, 0.3)
    np.testing.assert_allclose(b, a, rtol=1e-12, atol=1e-13)


def test_shared_latent_with_identity_factors_is_plain_attention():
    """R = d and B_Kh = B_Vh = I: the latents ARE the keys and values of every head; torch's attention on them."""
    import torch
    rng = np.random.default_rng(9)
    B, H, d, n = 1, 3, 8, 21
    c = O.LatentCache(B, 1, 32, d, "f32")
    c.k[:] = rng.standard_normal(c.k.shape).astype(np.float32); c.v[:] = rng.standard_normal(c.v.shape).astype(np.float32)
    c.seq_lens[:] = n
    q = rng.standard_normal((B, H, d))
    eye = np.broadcast_to(np.eye(d), (H, d, d)).copy()
    got = O.decode_attn_shared_latent(c, q, eye, eye, d ** -0.5)
    K = torch.from_numpy(c.k[0, 0, :n].astype(np.float64)); V = torch.from_numpy(c.v[0, 0, :n].astype(np.float64))
    want = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q[0])[:, None, :], K[None].expand(H, n, d),
                                                            V[None].expand(H, n, d))[:, 0].numpy()
    np.testing.assert_allclose(got[0], want, rtol=1e-10, atol=1e-12)


def test_shared_latent_int8_cache_reads_the_quantised_rows():
    """With an int8 cache the scheme attends over the dequantised codes (one scale per token for the whole rank-R row)."""
    rng = np.random.default_rng(10)
    B, H, R, d, n = 1, 2, 64, 16, 9
    c = O.LatentCache(B, 1, 64, R, "i8")
    lat = rng.standard_normal((1, n, R))
    c.store_rows("k", 0, 0, lat); c.store_rows("v", 0, 0, lat * 0.5); c.seq_lens[:] = n
    assert c.k_scale.shape == (1, 1, 64)
    BK = rng.standard_normal((H, R, d)); BV = rng.standard_normal((H, R, d)); q = rng.standard_normal((B, H, d))
    f = O.LatentCache(B, 1, 64, R, "f32")
    f.k[0, 0, :n] = (c.k[0, 0, :n].astype(np.float64) * c.k_scale[0, 0, :n].astype(np.float64)[:, None]).astype(np.float32)
    f.v[0, 0, :n] = (c.v[0, 0, :n].astype(np.float64) * c.v_scale[0, 0, :n].astype(np.float64)[:, None]).astype(np.float32)
    f.seq_lens[:] = n
    np.testing.assert_allclose(O.decode_attn_shared_latent(c, q, BK, BV, 0.2), O.decode_attn_shared_latent(f, q, BK, BV, 0.2),
                               rtol=1e-6, atol=1e-7)
    part = O.decode_attn_shared_latent(c, q, BK, BV, 0.2, heads=[(0, 1)])
    assert np.isnan(part[0, 0]).all() and np.array_equal(part[0, 1], O.decode_attn_shared_latent(c, q, BK, BV, 0.2)[0, 1])


def test_shared_latent_generators_are_seeded_and_shaped():
    import wsvd_inputs as WI
    sp = WI.spec("c3_small")
    BK, BV = WI.shared_up_factors(sp, 256)
    assert BK.shape == (sp.n_q_heads, 256, sp.d_head) and np.array_equal(BK, WI.shared_up_factors(sp, 256)[0])
    assert np.array_equal(BK, WI.bf16_exact(BK)) and not np.array_equal(BK, BV)
    a = WI.shared_latents(sp, 256, "k", 1, 10); b = WI.shared_latents(sp, 256, "v", 1, 10)
    assert a.shape == (10, 256) and a.dtype == np.float32 and not np.array_equal(a, b)
    assert np.array_equal(a, WI.shared_latents(sp, 256, "k", 1, 10))


@pytest.mark.parametrize("r,r_pad", [(115, 128), (77, 96), (5, 32)])
def test_zero_padded_rank_is_the_same_problem(r, r_pad):
    """A rank-r head run at a wider rank with zero columns in A and zero rows in B (how ranks between the supported
    widths reach the library): the quantiser sees the same abs-max and emits zero codes for the padding, and the
    attention result is the logical rank's (Section 3.1: K_h = C_h B_h only sums over the r latent channels)."""
    rng = np.random.default_rng(r)
    B, H, T, d, E = 2, 3, 37, 16, 48
    AK = rng.standard_normal((H, E, r)) / np.sqrt(E); AV = rng.standard_normal((H, E, r)) / np.sqrt(E)
    BK = rng.standard_normal((H, r, d)) / np.sqrt(r); BV = rng.standard_normal((H, r, d)) / np.sqrt(r)
    pad_a = lambda a: np.concatenate([a, np.zeros(a.shape[:-1] + (r_pad - r,))], axis=-1)
    pad_b = lambda b: np.concatenate([b, np.zeros((H, r_pad - r, d))], axis=1)
    caches = [O.LatentCache(B, H, T + 3, rr, "i8") for rr in (r, r_pad)]
    X = rng.standard_normal((T, B, E))
    for t in range(T):
        O.latent_append(caches[0], X[t], AK, AV)
        O.latent_append(caches[1], X[t], pad_a(AK), pad_a(AV))
    assert (caches[1].k[..., :r] == caches[0].k).all() and (caches[1].k[..., r:] == 0).all()
    assert (caches[1].v[..., :r] == caches[0].v).all() and (caches[1].v[..., r:] == 0).all()
    assert (caches[1].k_scale.view(np.uint16) == caches[0].k_scale.view(np.uint16)).all()
    assert (caches[1].v_scale.view(np.uint16) == caches[0].v_scale.view(np.uint16)).all()
    q = rng.standard_normal((B, H, d))
    o0 = O.decode_attn_reconstructed(caches[0], q, BK, BV, 0.25)
    o1 = O.decode_attn_reconstructed(caches[1], q, pad_b(BK), pad_b(BV), 0.25)
    assert np.abs(o0 - o1).max() <= 1e-13 * np.abs(o0).max()
