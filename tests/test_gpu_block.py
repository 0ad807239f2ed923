"""GPU parity of the quantised attention block (grouped-query layer with int4 weights and int8 activations,
Section 4.2): the W4A8 linear layer (integer accumulators bit-exact), the store of latents computed by it, and
the chain  quantise x -> W_Q / A_K / A_V -> store -> attention -> quantise o -> W_O  against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
from cases import build_block_case
from harness import DeviceLayer, as_dtype_dev, dev, err_stats, q_to_device
from test_gpu_parity import _append_compare, check_out, layer_for

pytestmark = pytest.mark.gpu


def gpu_linear(ctx, x_codes, x_scale, w_codes, w_scale):
    """numpy in, numpy out, through wsvd_linear_w4a8."""
    M, K = x_codes.shape
    N = w_codes.shape[0]
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    W.wsvd_linear_w4a8(ctx, dev(x_codes), dev(np.asarray(x_scale, np.float16).view(np.uint16)), dev(O.pack_w4(w_codes)),
                       dev(np.asarray(w_scale, np.float16).view(np.uint16)), M, K, N, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("M,K,N", [(1, 64, 32), (3, 192, 64), (16, 256, 32), (17, 320, 96), (32, 3584, 4096), (33, 512, 64),
                                   (48, 1792, 512), (64, 4096, 128), (32, 3584, 512)])
def test_linear_w4a8_integer_accumulators_bit_exact(M, K, N):
    """Unit scales: the fp32 output IS the int32 accumulator (|acc| < 2^24 for this data), so it must equal the
    oracle's int64 sum exactly.  Extreme codes (-128-free int8 range, -8 and 7 nibbles) are planted."""
    rng = np.random.default_rng(1000 * M + K + N)
    x = rng.integers(-127, 128, (M, K)).astype(np.int8)
    w = rng.integers(-8, 8, (N, K)).astype(np.int8)
    x[0, :] = 127; w[0, :] = -8; w[-1, :] = 7
    x[-1, ::2] = -127
    if K > 2048:                       # keep |acc| below 2^24 so the fp32 carrier is exact
        x[0, 2048:] = 0
    L = W.wsvd_create(0)
    got = gpu_linear(L, x, np.ones(M, np.float16), w, np.ones(N, np.float16))
    ref = O.linear_w4a8_int_accum(x, O.pack_w4(w))
    assert np.abs(ref).max() < 2 ** 24
    assert (got.astype(np.int64) == ref).all(), f"accumulators differ at {np.argwhere(got.astype(np.int64) != ref)[:5]}"
    W.wsvd_destroy(L)


def test_linear_w4a8_scaled_matches_oracle():
    c = build_block_case("c5_small")
    L = W.wsvd_create(0)
    for name, (wc, ws) in (("W_Q", c.wq), ("A_K", c.ak), ("A_V", c.av)):
        got = gpu_linear(L, c.x_codes, c.x_scale, wc, ws)
        ref = O.linear_w4a8(c.x_codes, c.x_scale, O.pack_w4(wc), ws)
        a, r, l2 = err_stats(got.astype(np.float64), ref)
        print(f"{name}: rel_max={r:.3e} rel_l2={l2:.3e}", flush=True)
        assert r <= 1e-6 and l2 <= 1e-6
    W.wsvd_destroy(L)


def test_linear_w4a8_split_equals_unsplit():
    rng = np.random.default_rng(3)
    M, K, N, N1 = 19, 448, 160, 96
    x = rng.integers(-127, 128, (M, K)).astype(np.int8)
    w = rng.integers(-8, 8, (N, K)).astype(np.int8)
    xs = (rng.random(M) + 0.5).astype(np.float16); ws = (rng.random(N) * 0.01 + 0.001).astype(np.float16)
    L = W.wsvd_create(0)
    whole = gpu_linear(L, x, xs, w, ws)
    a = torch.full((M, N1), float("nan"), dtype=torch.float32, device="cuda")
    b = torch.full((M, N - N1), float("nan"), dtype=torch.float32, device="cuda")
    u16 = lambda v: dev(np.asarray(v, np.float16).view(np.uint16))
    W.wsvd_linear_w4a8_split(L, dev(x), u16(xs), dev(O.pack_w4(w)), u16(ws), M, K, N, N1, a, b)
    torch.cuda.synchronize()
    assert (a.cpu().numpy() == whole[:, :N1]).all() and (b.cpu().numpy() == whole[:, N1:]).all()
    ref = O.linear_w4a8(x, xs, O.pack_w4(w), ws)
    assert np.abs(whole - ref).max() <= 1e-6 * np.abs(ref).max()
    for bad in (0, 48, N + 32):
        with pytest.raises(W.WsvdError) as e:
            W.wsvd_linear_w4a8_split(L, dev(x), u16(xs), dev(O.pack_w4(w)), u16(ws), M, K, N, bad, a, b)
        assert e.value.status == W.E_SHAPE
    W.wsvd_destroy(L)


def test_linear_w4a8_host_errors():
    L = W.wsvd_create(0)
    x = torch.zeros((4, 128), dtype=torch.int8, device="cuda")
    xs = torch.zeros(4, dtype=torch.int16, device="cuda")
    w = torch.zeros((32, 64), dtype=torch.uint8, device="cuda")
    ws = torch.zeros(32, dtype=torch.int16, device="cuda")
    out = torch.zeros((4, 32), dtype=torch.float32, device="cuda")
    for M, K, N in ((0, 128, 32), (65, 128, 32), (4, 96, 32), (4, 128, 48), (4, 131072, 32)):
        with pytest.raises(W.WsvdError) as e:
            W.wsvd_linear_w4a8(L, x, xs, w, ws, M, K, N, out)
        assert e.value.status == W.E_SHAPE
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_linear_w4a8(L, x, None, w, ws, 4, 128, 32, out)
    assert e.value.status == W.E_NULL
    W.wsvd_destroy(L)


@pytest.mark.parametrize("name,over", [("c5_small", dict()), ("c3_small", dict()), ("c4_small", dict()), ("c2_small", dict()),
                                       ("c1", dict(batch=3, context=70))], ids=["i8r64", "i8r32", "i4", "bf16", "f32"])
def test_latent_store_matches_oracle(name, over):
    """fp32 latents handed over with a leading dimension (as they sit in a fused projection's output)."""
    from cases import build_case
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    rng = np.random.default_rng(7)
    n_lat = sp.n_kv_heads * sp.rank
    ld = 2 * n_lat + 32
    buf = (rng.standard_normal((sp.batch, ld)) * np.exp(rng.standard_normal((sp.batch, 1)))).astype(np.float32)
    cK = buf[:, 16:16 + n_lat].reshape(sp.batch, sp.n_kv_heads, sp.rank)
    cV = buf[:, 16 + n_lat:16 + 2 * n_lat].reshape(sp.batch, sp.n_kv_heads, sp.rank)
    before = c.cache.seq_lens.copy()
    for b in range(sp.batch):
        n = int(before[b])
        c.cache.store_rows("k", b, n, cK[b][:, None, :].astype(np.float64))
        c.cache.store_rows("v", b, n, cV[b][:, None, :].astype(np.float64))
        c.cache.seq_lens[b] = n + 1
    d = dev(buf)
    W.wsvd_latent_store(L.ctx, L.desc, d[:, 16:], d[:, 16 + n_lat:], ld, L.cache)
    assert W.wsvd_check(L.ctx) == 0
    assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    flips = _append_compare(L, c.cache, cK.astype(np.float64), cV.astype(np.float64), before, sp.latent_dtype)
    assert flips == 0, "inputs are the same fp32 values on both sides: no rounding flip is legitimate"
    # untouched rows keep their content
    for plane, oc in ((0, c.cache.k), (1, c.cache.v)):
        gc, _, _ = L.download(plane, 0, int(before.min()))
        assert (gc.reshape(oc[:, :, :int(before.min())].shape) == oc[:, :, :int(before.min())]).all()
    # a full sequence is left alone and flagged
    L.seq_lens[0] = L.t_cap
    W.wsvd_latent_store(L.ctx, L.desc, d[:, 16:], d[:, 16 + n_lat:], ld, L.cache)
    assert W.wsvd_check(L.ctx) == W.E_CAPACITY
    lens = L.seq_lens.cpu().numpy()
    assert lens[0] == L.t_cap and (lens[1:] == c.cache.seq_lens[1:] + 1).all()
    L.close()


def _oracle_block(c, heads=None):
    sp = c.sp
    return O.attention_block_w4a8(c.cache, c.x_codes, c.x_scale, O.pack_w4(c.wq[0]), c.wq[1], O.pack_w4(c.ak[0]), c.ak[1],
                                  O.pack_w4(c.av[0]), c.av[1], c.BK.astype(np.float64), c.BV.astype(np.float64),
                                  O.pack_w4(c.wo[0]), c.wo[1], sp.n_q_heads, sp.d_head, c.sm_scale, heads=heads)


def _run_block(c, L, stagewise, ref=None, before=None, one_launch_store=False):
    """The GPU chain.  stagewise=True re-seeds every stage with the oracle's output of the previous one, so each
    stage is compared on identical inputs; False lets the GPU's own intermediates flow through.  one_launch_store
    (chained only): the store and the attention go through wsvd_decode_attn_store, as the benchmark's chain does."""
    sp = c.sp
    B, E, Hq, Hkv, d, r = sp.batch, sp.d_model, sp.n_q_heads, sp.n_kv_heads, sp.d_head, sp.rank
    u16 = lambda a: dev(np.asarray(a, np.float16).view(np.uint16))
    if ref is None:
        before = c.cache.seq_lens.copy()
        ref = _oracle_block(c)
    # 1. per-token int8 of the hidden state
    xq = torch.empty((B, E), dtype=torch.int8, device="cuda"); xs = torch.empty(B, dtype=torch.int16, device="cuda")
    W.wsvd_quantize_act_i8(L.ctx, dev(c.x32), W.F32, B, E, xq, xs)
    assert (xq.cpu().numpy() == c.x_codes).all() and (xs.cpu().numpy().view(np.float16) == c.x_scale).all()
    # 2. projections: W_Q, and A_K | A_V as one weight so that the latents land in one buffer
    q = torch.empty((B, Hq * d), dtype=torch.float32, device="cuda")
    lat = torch.empty((B, 2 * Hkv * r), dtype=torch.float32, device="cuda")
    akv = np.concatenate([c.ak[0], c.av[0]], 0); akv_s = np.concatenate([c.ak[1], c.av[1]])
    if stagewise:
        W.wsvd_linear_w4a8(L.ctx, xq, xs, dev(O.pack_w4(c.wq[0])), u16(c.wq[1]), B, E, Hq * d, q)
        W.wsvd_linear_w4a8(L.ctx, xq, xs, dev(O.pack_w4(akv)), u16(akv_s), B, E, 2 * Hkv * r, lat)
    else:                      # one launch over the stacked weight [W_Q; A_K; A_V], two outputs
        wall = np.concatenate([c.wq[0], akv], 0); wall_s = np.concatenate([c.wq[1], akv_s])
        W.wsvd_linear_w4a8_split(L.ctx, xq, xs, dev(O.pack_w4(wall)), u16(wall_s), B, E, Hq * d + 2 * Hkv * r, Hq * d, q, lat)
    torch.cuda.synchronize()
    for what, got, want in (("q", q.cpu().numpy(), ref["q"].reshape(B, -1)),
                            ("latents", lat.cpu().numpy(), np.concatenate([ref["cK"].reshape(B, -1), ref["cV"].reshape(B, -1)], 1))):
        a, rmax, l2 = err_stats(got.astype(np.float64), want)
        print(f"block {what}: rel_max={rmax:.3e} rel_l2={l2:.3e}", flush=True)
        assert rmax <= 1e-6 and l2 <= 1e-6
    # 3. store (one_launch_store: together with 4.)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    if one_launch_store:
        assert not stagewise
        L.out.fill_(float("nan"))
        W.wsvd_decode_attn_store(L.ctx, L.desc, lat, lat[:, Hkv * r:], 2 * Hkv * r, q.view(B, Hq, d), None, BKd, BVd, L.cache,
                                 int(before.max()) + 1, L.out)
        assert (L.seq_lens.cpu().numpy() == before + 1).all()
    else:
        W.wsvd_latent_store(L.ctx, L.desc, lat, lat[:, Hkv * r:], 2 * Hkv * r, L.cache)
    assert W.wsvd_check(L.ctx) == 0
    flips = _append_compare(L, c.cache, ref["cK"], ref["cV"], before, sp.latent_dtype)
    print(f"block store: boundary flips accepted = {flips}", flush=True)
    assert flips <= max(2, 2 * B * Hkv * r // 500)
    if stagewise:
        L.upload(c.cache)
    # 4. attention with the fp32 query as it left the projection
    qd = dev(ref["q"].astype(np.float32).reshape(B, Hq, d)) if stagewise else q.view(B, Hq, d)
    attn = L.out.cpu().numpy().astype(np.float64) if one_launch_store else L.attend(qd, None, BKd, BVd, int(c.cache.seq_lens.max()))
    check_out(attn, ref["attn"], "i8", f"block attention ({'stagewise' if stagewise else 'chained'})")
    # 5. int8 of the attention output, W_O
    o_in = dev(ref["attn"].reshape(B, Hq * d).astype(np.float32)) if stagewise else L.out.view(B, Hq * d)
    oq = torch.empty((B, Hq * d), dtype=torch.int8, device="cuda"); osc = torch.empty(B, dtype=torch.int16, device="cuda")
    W.wsvd_quantize_act_i8(L.ctx, o_in, W.F32, B, Hq * d, oq, osc)
    y = torch.empty((B, E), dtype=torch.float32, device="cuda")
    W.wsvd_linear_w4a8(L.ctx, oq, osc, dev(O.pack_w4(c.wo[0])), u16(c.wo[1]), B, Hq * d, E, y)
    torch.cuda.synchronize()
    if stagewise:
        assert (oq.cpu().numpy() == ref["o_codes"]).all() and (osc.cpu().numpy().view(np.float16) == ref["o_scale"]).all()
    a, rmax, l2 = err_stats(y.cpu().numpy().astype(np.float64), ref["y"])
    print(f"block y ({'stagewise' if stagewise else 'chained'}): max_abs={a:.3e} rel_max={rmax:.3e} rel_l2={l2:.3e}", flush=True)
    if stagewise:
        assert rmax <= 1e-6 and l2 <= 1e-6
    else:
        # the chained run re-quantises the GPU's own attention output: a code may differ from the oracle's by one
        # step where the fp32 result sits on a rounding boundary, which the bars for the integer paths cover
        assert a <= 2e-2 and l2 <= 1e-3


@pytest.mark.parametrize("stagewise,one_launch", [(True, False), (False, False), (False, True)],
                         ids=["stagewise", "chained", "chained-store-and-attend"])
def test_block_c5_small(stagewise, one_launch):
    c = build_block_case("c5_small")
    L = layer_for(c); L.upload(c.cache)
    _run_block(c, L, stagewise, one_launch_store=one_launch)
    L.close()


@pytest.mark.parametrize("name", ["c5_small", "c3_small", "c4_small"])
def test_store_and_attend_equals_the_two_calls(name):
    """wsvd_decode_attn_store against wsvd_latent_store + wsvd_decode_attn on a twin layer: the same cache bytes and
    lengths afterwards; outputs within the bars of the oracle (a single launch attends the new row's tile last, so
    the sums differ in order) and of each other.  c5_small takes the single-launch kernel (7 query heads per kv
    head), the other two the two-launch route of the same entry point.  Ragged lengths, one sequence on a tile edge,
    one empty, one full."""
    from cases import build_case
    c = build_case(name)
    sp = c.sp
    lens = c.cache.seq_lens.copy()
    lens[0] = 64 if sp.batch > 1 else lens[0]                 # the new row opens a tile
    if sp.batch > 2:
        lens[1] = 0                                            # the new row is the only one
    c.cache.seq_lens[:] = lens
    rng = np.random.default_rng(11)
    n_lat = sp.n_kv_heads * sp.rank
    lat = (rng.standard_normal((sp.batch, 2 * n_lat)) * 0.7).astype(np.float32)
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    outs, caches = [], []
    for fused in (False, True):
        L = layer_for(c); L.upload(c.cache)
        d = dev(lat)
        n_max = int(lens.max()) + 1
        if fused:
            L.out.fill_(float("nan"))
            W.wsvd_decode_attn_store(L.ctx, L.desc, d, d[:, n_lat:], 2 * n_lat, qd, qs, BKd, BVd, L.cache, n_max, L.out)
            torch.cuda.synchronize()
            o = L.out.cpu().numpy().astype(np.float64)
        else:
            W.wsvd_latent_store(L.ctx, L.desc, d, d[:, n_lat:], 2 * n_lat, L.cache)
            o = L.attend(qd, qs, BKd, BVd, n_max)
        assert W.wsvd_check(L.ctx) == 0
        assert (L.seq_lens.cpu().numpy() == lens + 1).all()
        outs.append(o)
        caches.append([L.download(pl, 0, n_max) for pl in (0, 1)])
        if fused:                                              # a full sequence is left alone, attended as it is, and flagged
            L.seq_lens[0] = L.t_cap
            W.wsvd_decode_attn_store(L.ctx, L.desc, d, d[:, n_lat:], 2 * n_lat, qd, qs, BKd, BVd, L.cache, L.t_cap, L.out)
            assert W.wsvd_check(L.ctx) == W.E_CAPACITY
            after = L.seq_lens.cpu().numpy()
            assert after[0] == L.t_cap and (after[1:] == lens[1:] + 2).all()
        L.close()
    for pl in (0, 1):
        for a, b in zip(caches[0][pl], caches[1][pl]):
            if a is not None:
                for bi in range(sp.batch):                     # rows below each sequence's new length
                    n = int(lens[bi]) + 1
                    assert (np.asarray(a)[bi, :, :n].tobytes() == np.asarray(b)[bi, :, :n].tobytes()), (name, pl, bi)
    # oracle: the same store, then the definition
    for b in range(sp.batch):
        n = int(lens[b])
        c.cache.store_rows("k", b, n, lat[b, :n_lat].reshape(sp.n_kv_heads, 1, sp.rank).astype(np.float64))
        c.cache.store_rows("v", b, n, lat[b, n_lat:].reshape(sp.n_kv_heads, 1, sp.rank).astype(np.float64))
        c.cache.seq_lens[b] = n + 1
    ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    for o, what in zip(outs, ("two calls", "one call")):
        check_out(o, ref, sp.latent_dtype, f"store and attend, {name}, {what}")
    assert np.abs(outs[0] - outs[1]).max() <= 1e-4 * max(np.abs(ref).max(), 1e-30)


@pytest.mark.parametrize("layer", list(range(28)))
def test_config5_block_full_size(layer):
    """Every one of the 28 independent layers of the workload (per-layer seeds for weights, factors and cache, the same
    hidden state fed to each) at its real shape: batch 32, 28 query / 4 kv heads, rank 64, 8192 rows of context, the
    launches the benchmark times.  The reconstructing oracle runs on a sample of heads (96 for layer 3, 12 elsewhere);
    the absorbed oracle, checked against it on that sample, provides every head, from which the oracle's own quantiser
    and W_O give the reference block output."""
    import time
    t0 = time.time()
    c = build_block_case("c5", layer=layer)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    rng = np.random.default_rng(5 + layer)
    n_sample = 96 if layer == 3 else 12
    heads = [(int(b), int(h)) for b, h in zip(rng.integers(0, sp.batch, n_sample), rng.integers(0, sp.n_q_heads, n_sample))]
    before = c.cache.seq_lens.copy()
    ref = _oracle_block(c, heads=heads)
    q32 = ref["q"].astype(np.float32).astype(np.float64)
    attn_all = O.decode_attn_absorbed(c.cache, q32, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    m = ~np.isnan(ref["attn"])
    assert m.sum() >= (n_sample * 2 // 3) * sp.d_head          # the draws contain a few repeats
    assert np.abs(attn_all[m] - ref["attn"][m]).max() <= 1e-9 * np.abs(ref["attn"][m]).max()
    ref["attn"] = attn_all
    ref["o_codes"], ref["o_scale"] = O.quantize_act_i8(attn_all.reshape(sp.batch, -1).astype(np.float32))
    ref["y"] = O.linear_w4a8(ref["o_codes"], ref["o_scale"], O.pack_w4(c.wo[0]), c.wo[1])
    print(f"c5 layer {layer}: inputs and oracle in {time.time() - t0:.1f}s", flush=True)
    _run_block(c, L, False, ref=ref, before=before, one_launch_store=(layer % 2 == 1))    # odd layers: as the benchmark's chain
    L.close()
