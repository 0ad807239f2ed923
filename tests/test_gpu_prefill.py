"""GPU parity tests for the prefill of the cache: consecutive tokens of one sequence projected, stored and counted in
chunks of up to 64 (wsvd_prefill_append), against the oracle's ``latent_prefill``."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
import wsvd_inputs as WI
from cases import build_case
from harness import as_dtype_dev, check_i8_rows, q_to_device
from test_gpu_parity import check_out, layer_for, run_attend

pytestmark = pytest.mark.gpu


def _big_workspace(L, n_tokens=64):
    """A workspace that also serves a chunk of n_tokens rows (sized with a descriptor whose batch is n_tokens)."""
    d64 = type(L.desc).from_buffer_copy(L.desc)
    d64.batch = n_tokens
    need = max(W.wsvd_workspace_bytes(d64), W.wsvd_workspace_bytes(L.desc))
    L.ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    W.wsvd_set_workspace(L.ctx, L.ws)


def _latents64(X, A):
    """fp64 latents [Hkv, n, r] of the rows X [n, E] (what the oracle quantises)."""
    return np.transpose(O.project_latents(np.asarray(X, np.float64), np.asarray(A, np.float64)), (1, 0, 2))


def _compare_rows(L, oc, b, t0, n, dtype, cK64, cV64):
    """Rows [t0, t0 + n) of sequence b, both planes, against the oracle's cache.  cK64 / cV64 [Hkv, n, r] are the
    oracle's fp64 latents of those rows.  A stored value may differ from the oracle's only by one step and only where
    the fp64 value sits on a rounding boundary of the storage format (the GPU sums in fp32, in another order); every
    row is compared, also those whose scale moved.  Returns the number of accepted differences."""
    flips = 0
    for plane, codes, c64 in ((0, oc.k, cK64), (1, oc.v, cV64)):
        gc, gs, _ = L.download(plane, t0, n)
        gc = gc[b]; want = codes[b, :, t0:t0 + n]
        c64 = np.asarray(c64, np.float64)[:, :n]
        if dtype == "f32":
            np.testing.assert_allclose(gc.view(np.float32).reshape(want.shape), want, rtol=2e-5, atol=1e-6)
        elif dtype == "bf16":
            gb = gc.view(np.uint16).reshape(want.shape)
            bad = gb != want
            if bad.any():
                assert np.abs(gb.astype(np.int32) - want.astype(np.int32))[bad].max() == 1, "bf16 latents differ by more than one step"
                gv = O.f64_from_bf16_bits(gb[bad]); ov = O.f64_from_bf16_bits(want[bad])
                dist = np.abs(c64[bad] - 0.5 * (gv + ov))          # distance of the exact value from the rounding boundary
                assert (dist <= 1e-3 * np.abs(gv - ov) + 1e-6 * np.abs(c64).max()).all(), \
                    "bf16 latent differs away from a rounding boundary"
            flips += int(bad.sum())
        else:
            flips += check_i8_rows(gc.reshape(want.shape), gs[b].reshape(want.shape[:-1]), c64,
                                   f"prefill rows b={b} plane={plane}")
    return flips


@pytest.mark.parametrize("name,over", [("c3_small", dict()), ("c2_small", dict()), ("c1", dict(batch=2, context=70)),
                                       ("c5_small", dict()), ("c3_small", dict(rank=64))], ids=["i8", "bf16", "f32", "i8r64g7", "i8r64"])
def test_prefill_matches_oracle(name, over):
    c = build_case(name, extra_cap=256, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    xdt = "f32" if sp.factor_dtype == "f32" else "bf16"
    b = sp.batch - 1
    n_total = 150
    X = WI.hidden_states(sp, n_total, 1.0, which="ctx", sub=77)
    if xdt == "bf16":
        X = WI.bf16_exact(X)
    AKd, AVd = L.pack_A(c.AK, sp.factor_dtype), L.pack_A(c.AV, sp.factor_dtype)
    xd = as_dtype_dev(X, xdt)
    n0 = int(c.cache.seq_lens[b])
    others = c.cache.seq_lens.copy()
    # the layer's workspace was sized for its own batch: a 64-token chunk needs more, and says so
    if sp.batch < 64:
        with pytest.raises(W.WsvdError) as e:
            W.wsvd_prefill_append(L.ctx, L.desc, xd, None, 64, b, AKd, AVd, L.cache)
        assert e.value.status == W.E_WORKSPACE
    _big_workspace(L)
    assert not O.latent_prefill(c.cache, b, X.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    for i0, n in ((0, 64), (64, 64), (128, 22)):
        W.wsvd_prefill_append(L.ctx, L.desc, xd[i0:i0 + n], None, n, b, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == 0
    others[b] = n0 + n_total
    assert (L.seq_lens.cpu().numpy() == others).all() and (c.cache.seq_lens == others).all()
    flips = _compare_rows(L, c.cache, b, n0, n_total, sp.latent_dtype, _latents64(X, c.AK), _latents64(X, c.AV))
    print(f"prefill {name}: one-step differences accepted = {flips}", flush=True)
    # rows of the other sequences and the old rows of this one are untouched
    m = int(min(others.min(), n0))
    for plane, codes in ((0, c.cache.k), (1, c.cache.v)):
        gc, _, _ = L.download(plane, 0, m)
        assert (gc.reshape(codes[:, :, :m].shape) == codes[:, :, :m]).all()
    # attention over the prefilled cache (GPU rows on the GPU side, oracle rows on the oracle side)
    got, ref = run_attend(c, L)
    check_out(got, ref, sp.latent_dtype, f"attention after prefill, {name}")
    L.close()


def test_prefill_capacity_int4_and_arguments():
    c = build_case("c3_small", extra_cap=0)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    _big_workspace(L)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    X = WI.bf16_exact(WI.hidden_states(sp, 64, 1.0, which="ctx", sub=5))
    xd = as_dtype_dev(X, "bf16")
    b = 0
    n0 = int(c.cache.seq_lens[b]); room = L.t_cap - n0
    assert 0 < room < 64
    assert O.latent_prefill(c.cache, b, X.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    W.wsvd_prefill_append(L.ctx, L.desc, xd, None, 64, b, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == W.E_CAPACITY
    assert int(L.seq_lens[b]) == L.t_cap
    _compare_rows(L, c.cache, b, n0, room, "i8", _latents64(X, c.AK), _latents64(X, c.AV))   # the rows that fitted are there
    W.wsvd_prefill_append(L.ctx, L.desc, xd, None, 3, b, AKd, AVd, L.cache)   # a full sequence: nothing stored, reported
    assert W.wsvd_check(L.ctx) == W.E_CAPACITY and int(L.seq_lens[b]) == L.t_cap
    for bad_n, bad_b in ((0, 0), (4, -2), (4, sp.batch)):
        with pytest.raises(W.WsvdError) as e:
            W.wsvd_prefill_append(L.ctx, L.desc, xd, None, bad_n, bad_b, AKd, AVd, L.cache)
        assert e.value.status == W.E_SHAPE
    L.close()


@pytest.mark.parametrize("name,over", [("c3_small", dict()), ("c5_small", dict()), ("c3_small", dict(rank=64, batch=2, context=45))],
                         ids=["i8", "i8r64g7", "i8r64"])
def test_prefill_whole_prompt_projection_matches_oracle(name, over):
    """More than 64 tokens in one call: the tiled projection (int8 latents, bf16 hidden states and factors)."""
    c = build_case(name, extra_cap=320, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    b = sp.batch - 1
    n_total = 150 + 33 + 1
    X = WI.bf16_exact(WI.hidden_states(sp, n_total, 1.0, which="ctx", sub=78))
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    xd = as_dtype_dev(X, "bf16")
    n0 = int(c.cache.seq_lens[b])
    others = c.cache.seq_lens.copy()
    assert not O.latent_prefill(c.cache, b, X.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    W.wsvd_prefill_append(L.ctx, L.desc, xd[:150], None, 150, b, AKd, AVd, L.cache)       # 4 full tiles and a ragged one
    W.wsvd_ctx_set_option(L.ctx, "prefill_tiled", 1)                                                  # short chunks on the same kernel
    try:
        W.wsvd_prefill_append(L.ctx, L.desc, xd[150:183], None, 33, b, AKd, AVd, L.cache)
        W.wsvd_prefill_append(L.ctx, L.desc, xd[183:], None, 1, b, AKd, AVd, L.cache)
    finally:
        W.wsvd_ctx_set_option(L.ctx, "prefill_tiled", 0)
    assert W.wsvd_check(L.ctx) == 0
    others[b] = n0 + n_total
    assert (L.seq_lens.cpu().numpy() == others).all() and (c.cache.seq_lens == others).all()
    flips = _compare_rows(L, c.cache, b, n0, n_total, "i8", _latents64(X, c.AK), _latents64(X, c.AV))
    print(f"tiled projection {name}: one-step differences accepted = {flips}", flush=True)
    m = int(min(others.min(), n0))
    for plane, codes in ((0, c.cache.k), (1, c.cache.v)):
        gc, _, _ = L.download(plane, 0, m)
        assert (gc.reshape(codes[:, :, :m].shape) == codes[:, :, :m]).all()
    got, ref = run_attend(c, L)
    check_out(got, ref, "i8", f"attention after the tiled projection, {name}")
    L.close()


@pytest.mark.parametrize("name,over,shape,n", [("c3_small", {}, 0, 100), ("c3_small", {}, 1, 100), ("c3_small", {}, 44, 100),
                                               ("c3_small", {}, 42, 100), ("c3_small", {}, 24, 100), ("c3_small", dict(rank=64), 1, 100),
                                               ("c5_small", {}, 1, 300), ("c3_small", dict(batch=2, context=40), 1, 515),
                                               ("c3_small", {}, 2, 100), ("c5_small", {}, 2, 300),
                                               ("c3_small", dict(batch=2, context=40, rank=64), 2, 515)],
                         ids=["auto", "staged", "d44", "d42", "d24", "staged-r64", "staged-r64g7-300", "staged-515",
                              "staged8", "staged8-r64g7-300", "staged8-r64-515"])
def test_prefill_all_sequences_in_one_call(name, over, shape, n):
    """seq_index = -1: the same number of prompt tokens for every sequence, x = [batch, n_tokens, d_model]; the staged
    projection kernel and every wave-tile shape of the direct one."""
    c = build_case(name, extra_cap=n + 92, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    X = np.stack([WI.bf16_exact(WI.hidden_states(sp, n, 1.0, which="ctx", sub=40 + b)) for b in range(sp.batch)])
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    xd = as_dtype_dev(X.reshape(sp.batch * n, -1), "bf16")
    starts = c.cache.seq_lens.copy()
    for b in range(sp.batch):
        assert not O.latent_prefill(c.cache, b, X[b].astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    W.wsvd_ctx_set_option(L.ctx, "project_shape", shape)
    try:
        W.wsvd_prefill_append(L.ctx, L.desc, xd, None, n, -1, AKd, AVd, L.cache)
    finally:
        W.wsvd_ctx_set_option(L.ctx, "project_shape", 0)
    assert W.wsvd_check(L.ctx) == 0
    assert (L.seq_lens.cpu().numpy() == starts + n).all()
    flips = sum(_compare_rows(L, c.cache, b, int(starts[b]), n, "i8", _latents64(X[b], c.AK), _latents64(X[b], c.AV))
                for b in range(sp.batch))
    print(f"all sequences, shape {shape}: one-step differences accepted = {flips}", flush=True)
    m = int(starts.min())
    for plane, codes in ((0, c.cache.k), (1, c.cache.v)):
        gc, _, _ = L.download(plane, 0, m)
        assert (gc.reshape(codes[:, :, :m].shape) == codes[:, :, :m]).all()
    got, ref = run_attend(c, L)
    check_out(got, ref, "i8", f"attention after the projection of all sequences, shape {shape}")
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_prefill_append(L.ctx, L.desc, xd, None, n, -2, AKd, AVd, L.cache)
    assert e.value.status == W.E_SHAPE
    L.close()


def test_prefill_whole_prompt_projection_capacity_and_formats():
    c = build_case("c3_small", extra_cap=70)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    X = WI.bf16_exact(WI.hidden_states(sp, 200, 1.0, which="ctx", sub=6))
    xd = as_dtype_dev(X, "bf16")
    b = int(np.argmax(c.cache.seq_lens))
    n0 = int(c.cache.seq_lens[b]); room = L.t_cap - n0
    assert 64 < room < 200
    before = L.seq_lens.cpu().numpy().copy()
    assert O.latent_prefill(c.cache, b, X.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    W.wsvd_prefill_append(L.ctx, L.desc, xd, None, 200, b, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == W.E_CAPACITY
    before[b] = L.t_cap
    assert (L.seq_lens.cpu().numpy() == before).all()
    _compare_rows(L, c.cache, b, n0, room, "i8", _latents64(X, c.AK), _latents64(X, c.AV))   # the rows that fitted are there
    snap = L.download(0, 0, L.t_cap)[0].copy()
    W.wsvd_prefill_append(L.ctx, L.desc, xd, None, 100, b, AKd, AVd, L.cache)   # a full sequence: nothing stored, reported
    assert W.wsvd_check(L.ctx) == W.E_CAPACITY and int(L.seq_lens[b]) == L.t_cap
    assert (L.download(0, 0, L.t_cap)[0] == snap).all()
    L.close()
    # float latents take at most 64 tokens per call (int4 goes through the tiled projection: test_prefill_int4_tiled)
    for name in ("c2_small",):
        c2 = build_case(name, extra_cap=128)
        L2 = layer_for(c2); L2.upload(c2.cache)
        with pytest.raises(W.WsvdError) as e:
            W.wsvd_prefill_append(L2.ctx, L2.desc, xd, None, 65, 0, AKd, AVd, L2.cache)
        assert e.value.status == W.E_SHAPE
        L2.close()


# ------------------------------------------------------------------------------------------ attention over the prompt
def _multi_q(c, nq, seed=9):
    """Queries of nq tokens per sequence in the layout [B, Hkv, nq, G, d], bf16-exact."""
    sp = c.sp
    G = sp.n_q_heads // sp.n_kv_heads
    rng = np.random.default_rng(seed)
    return WI.bf16_exact(rng.standard_normal((sp.batch, sp.n_kv_heads, nq, G, sp.d_head)).astype(np.float32))


def _prefill_attn(L, c, q32, nq, n_after, max_len, q_dtype="bf16"):
    sp = c.sp
    G = sp.n_q_heads // sp.n_kv_heads
    d = type(L.desc).from_buffer_copy(L.desc)
    d.q_dtype = W.DTYPES[q_dtype]
    if nq * G <= 8:        # the slot kernel merges context splits through the workspace; the tiled kernel needs none
        dws = type(d).from_buffer_copy(d); dws.n_q_heads = sp.n_kv_heads * nq * G
        L.ws = torch.empty(max(W.wsvd_workspace_bytes(dws), W.wsvd_workspace_bytes(L.desc)), dtype=torch.uint8, device="cuda")
        W.wsvd_set_workspace(L.ctx, L.ws)
    out = torch.full(q32.shape, float("nan"), dtype=torch.float32, device="cuda")
    W.wsvd_prefill_attn(L.ctx, d, as_dtype_dev(q32, q_dtype), nq, n_after, as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16"),
                        L.cache, max_len, out)
    assert W.wsvd_check(L.ctx) == 0
    return out.cpu().numpy().astype(np.float64)


MULTI_CASES = [
    ("c3_small", 8, 0, dict()),                                     # 8 tokens of one head per kv head
    ("c3_small", 5, 0, dict(context=2000, batch=2)),                # several chunks of context
    ("c3_small", 4, 11, dict(n_q_heads=8, n_kv_heads=4)),           # 4 tokens x 2 heads, 11 later rows in the cache
    ("c3_small", 1, 0, dict(n_q_heads=16, n_kv_heads=2)),           # one token: the decode case through this entry
    ("c5_small", 1, 0, dict()),                                     # rank 64, 7 heads per kv head
    ("c3_small", 8, 64, dict(rank=64, context=700)),                # a full tile of later rows
    ("c3_small", 3, 0, dict(context=130, q="f32")),
]


@pytest.mark.parametrize("name,nq,n_after,over", MULTI_CASES, ids=[f"{n}-nq{q}-after{a}-{'-'.join(f'{k}{v}' for k, v in o.items())}" for n, q, a, o in MULTI_CASES])
def test_prefill_attention_matches_oracle(name, nq, n_after, over):
    over = dict(over)
    qd = over.pop("q", "bf16")
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    q32 = _multi_q(c, nq)
    got = _prefill_attn(L, c, q32, nq, n_after, int(c.cache.seq_lens.max()), qd)
    ref = O.causal_attn_reconstructed(c.cache, q32.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64),
                                      c.sm_scale, n_after=n_after)
    check_out(got, ref, "i8", f"prefill attention {name} nq={nq} n_after={n_after} {over}")
    if nq > 1:      # the tokens really see different prefixes: dropping the mask would change the first token's output
        full = O.causal_attn_reconstructed(c.cache, q32[:, :, :1].astype(np.float64), c.BK.astype(np.float64),
                                           c.BV.astype(np.float64), c.sm_scale, n_after=n_after)
        assert np.abs(full - ref[:, :, :1]).max() > 1e-4
    L.close()


def test_prefill_attention_short_sequences_and_errors():
    """Sequences shorter than the token block (some tokens before the start), an empty one, lengths around tile edges."""
    lens = [0, 1, 3, 8, 63, 64, 65, 66, 127, 128, 129, 200]
    c = build_case("c3_small", batch=len(lens), context=200, ragged=(), extra_cap=0, steps=1)
    for b, n in enumerate(lens):
        c.cache.seq_lens[b] = n
    L = layer_for(c); L.upload(c.cache)
    nq = 4
    q32 = _multi_q(c, nq)
    got = _prefill_attn(L, c, q32, nq, 0, 200)
    ref = O.causal_attn_reconstructed(c.cache, q32.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    assert (got[0] == 0).all() and (got[1, :, :3] == 0).all() and (got[2, :, :1] == 0).all()
    check_out(got, ref, "i8", "prefill attention, short sequences")
    d = L.desc
    qd = as_dtype_dev(q32, "bf16")
    out = torch.empty(q32.shape, dtype=torch.float32, device="cuda")
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    with pytest.raises(W.WsvdError) as e:            # the layer's own query type is int8
        W.wsvd_prefill_attn(L.ctx, d, qd, nq, 0, BKd, BVd, L.cache, 200, out)
    assert e.value.status == W.E_DTYPE
    d2 = type(d).from_buffer_copy(d); d2.q_dtype = W.DTYPES["bf16"]
    d3 = type(d).from_buffer_copy(d); d3.q_dtype = W.DTYPES["f32"]
    with pytest.raises(W.WsvdError) as e:            # more than 8 query rows per kv head: bf16 queries only
        W.wsvd_prefill_attn(L.ctx, d3, qd, 9, 0, BKd, BVd, L.cache, 200, out)
    assert e.value.status == W.E_UNSUPPORTED
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_prefill_attn(L.ctx, d2, qd, 0, 0, BKd, BVd, L.cache, 200, out)
    assert e.value.status == W.E_SHAPE
    L.close()


def test_prompt_prefill_end_to_end():
    """A 150-token prompt: cache built in chunks of 64, attention of all its tokens in blocks of 8 with the later rows
    already in the cache; every token's output against the oracle's causal attention over the oracle's own cache."""
    c = build_case("c3_small", batch=2, context=37, extra_cap=256)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    _big_workspace(L)
    b, n_total = 1, 150
    X = WI.bf16_exact(WI.hidden_states(sp, n_total, 1.0, which="ctx", sub=3))
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    xd = as_dtype_dev(X, "bf16")
    O.latent_prefill(c.cache, b, X.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    for i0 in range(0, n_total, 64):
        n = min(64, n_total - i0)
        W.wsvd_prefill_append(L.ctx, L.desc, xd[i0:i0 + n], None, n, b, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == 0
    n_end = int(c.cache.seq_lens[b])
    rng = np.random.default_rng(12)
    q_all = WI.bf16_exact(rng.standard_normal((sp.n_kv_heads, n_total, 1, sp.d_head)).astype(np.float32))   # [Hkv, tokens, G=1, d]
    worst = 0.0
    for i0 in (0, 8, 64, 136, 142):               # blocks at the start, across the chunk edge, and the ragged end
        nq = min(8, n_total - i0)
        n_after = n_total - i0 - nq
        q32 = np.zeros((sp.batch, sp.n_kv_heads, nq, 1, sp.d_head), np.float32)
        q32[b] = q_all[:, i0:i0 + nq]
        got = _prefill_attn(L, c, q32, nq, n_after, n_end)
        # sequence 0 is shorter than n_after: all its tokens are before its start
        ref = O.causal_attn_reconstructed(c.cache, q32.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64),
                                          c.sm_scale, n_after=n_after)
        assert (got[0] == 0).all() or int(c.cache.seq_lens[0]) > n_after
        check_out(got[b:b + 1], ref[b:b + 1], "i8", f"prompt tokens {i0}..{i0 + nq - 1}")
    L.close()


# ------------------------------------------------------------------------------------------ tiled kernel (any n_q)
TILED_CASES = [
    ("c3_small", 32, 0, dict()),                                    # exactly one block of query rows
    ("c3_small", 333, 0, dict()),                                   # the whole sequence as the prompt
    ("c3_small", 50, 7, dict(context=2000, batch=2)),               # ragged last block, later rows in the cache
    ("c3_small", 40, 0, dict(n_q_heads=8, n_kv_heads=4)),           # two heads per kv head: 80 query rows
    ("c5_small", 20, 3, dict()),                                    # rank 64, seven heads per kv head: 140 rows
    ("c3_small", 64, 64, dict(rank=64, context=700)),
    ("c3_small", 9, 0, dict(d_head=64)),                            # head dim 64
]


@pytest.mark.parametrize("name,nq,n_after,over", TILED_CASES, ids=[f"{n}-nq{q}-after{a}-{'-'.join(f'{k}{v}' for k, v in o.items())}" for n, q, a, o in TILED_CASES])
def test_prefill_attention_tiled_matches_oracle(name, nq, n_after, over):
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    q32 = _multi_q(c, nq, seed=21)
    got = _prefill_attn(L, c, q32, nq, n_after, int(c.cache.seq_lens.max()))
    ref = O.causal_attn_reconstructed(c.cache, q32.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64),
                                      c.sm_scale, n_after=n_after)
    check_out(got, ref, "i8", f"tiled prefill attention {name} nq={nq} n_after={n_after} {over}")
    L.close()


def test_prefill_attention_tiled_equals_slot_kernel_and_handles_short_sequences():
    lens = [0, 1, 3, 8, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200]
    c = build_case("c3_small", batch=len(lens), context=200, ragged=(), extra_cap=0, steps=1)
    for b, n in enumerate(lens):
        c.cache.seq_lens[b] = n
    L = layer_for(c); L.upload(c.cache)
    # 40 tokens: most sequences are shorter than the block, many tokens sit before the start
    q32 = _multi_q(c, 40, seed=5)
    got = _prefill_attn(L, c, q32, 40, 0, 200)
    ref = O.causal_attn_reconstructed(c.cache, q32.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    assert (got[0] == 0).all() and (got[2, :, :37] == 0).all()
    check_out(got, ref, "i8", "tiled prefill attention, short sequences")
    # up to 8 slots both kernels apply: same result within the int8 bar of each against the oracle, and close to each other
    q8 = _multi_q(c, 6, seed=6)
    a = _prefill_attn(L, c, q8, 6, 2, 200)
    W.wsvd_ctx_set_option(L.ctx, "prefill_tiled", 1)
    try:
        t = _prefill_attn(L, c, q8, 6, 2, 200)
    finally:
        W.wsvd_ctx_set_option(L.ctx, "prefill_tiled", 0)
    ref8 = O.causal_attn_reconstructed(c.cache, q8.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale, n_after=2)
    check_out(t, ref8, "i8", "tiled kernel, 6 tokens")
    check_out(a, ref8, "i8", "slot kernel, 6 tokens")
    # the two kernels agree to the tiled one's operand rounding (fp16 values and weights: 2^-12 relative each)
    assert np.abs(a - t).max() < 1e-3 * np.abs(ref8).max()
    L.close()


def test_whole_prompt_in_one_call():
    """Cache built in chunks of 64, then the attention of all 150 prompt tokens in a single launch."""
    c = build_case("c3_small", batch=2, context=37, extra_cap=256)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    _big_workspace(L)
    b, n_total = 1, 150
    X = WI.bf16_exact(WI.hidden_states(sp, n_total, 1.0, which="ctx", sub=3))
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    xd = as_dtype_dev(X, "bf16")
    O.latent_prefill(c.cache, b, X.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    for i0 in range(0, n_total, 64):
        n = min(64, n_total - i0)
        W.wsvd_prefill_append(L.ctx, L.desc, xd[i0:i0 + n], None, n, b, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == 0
    q32 = _multi_q(c, n_total, seed=13)
    got = _prefill_attn(L, c, q32, n_total, 0, int(c.cache.seq_lens.max()))
    ref = O.causal_attn_reconstructed(c.cache, q32.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    # sequence 0 holds 37 rows: its last 37 query tokens see a prefix, the first 113 sit before its start
    assert (got[0, :, :113] == 0).all() and np.abs(got[0, :, 113:]).min() > 0
    check_out(got, ref, "i8", "whole prompt, one launch")
    L.close()


def test_prefill_full_size_sampled():
    """The batched int8 workload's shape in the launch configuration the benchmark times: the cache of all 16 x 2048
    prompt tokens in one launch, then the attention of all of them in one launch.  The oracle builds the cache of two
    of the sequences itself and computes a sample of their tokens' outputs."""
    c = build_case("c3")
    sp = c.sp
    T = sp.context
    G = sp.n_q_heads // sp.n_kv_heads
    L = layer_for(c)
    L.seq_lens.zero_()
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    X = np.stack([WI.bf16_exact(WI.hidden_states(sp, T, 1.0, which="ctx", sub=100 + b)) for b in range(sp.batch)])
    xd = as_dtype_dev(X.reshape(sp.batch * T, -1), "bf16")
    print("full-size prefill: projection launch", flush=True)
    W.wsvd_prefill_append(L.ctx, L.desc, xd, None, T, -1, AKd, AVd, L.cache)
    torch.cuda.synchronize()
    assert W.wsvd_check(L.ctx) == 0 and (L.seq_lens.cpu().numpy() == T).all()
    seqs = [0, sp.batch - 1]
    oc = O.LatentCache(sp.batch, sp.n_kv_heads, L.t_cap, sp.rank, "i8")
    AK64, AV64 = c.AK.astype(np.float64), c.AV.astype(np.float64)
    flips = 0
    for b in seqs:
        assert not O.latent_prefill(oc, b, X[b].astype(np.float64), AK64, AV64)
        flips += _compare_rows(L, oc, b, 0, T, "i8", _latents64(X[b], c.AK), _latents64(X[b], c.AV))
    print(f"full-size prefill: one-step differences accepted in 2 x {T} x {sp.n_kv_heads} rows = {flips}", flush=True)
    # attention of the whole prompt
    rng = np.random.default_rng(77)
    q32 = WI.bf16_exact(rng.standard_normal((sp.batch, sp.n_kv_heads, T, G, sp.d_head), dtype=np.float32))
    d = type(L.desc).from_buffer_copy(L.desc)
    d.q_dtype = W.DTYPES["bf16"]
    out = torch.full(q32.shape, float("nan"), dtype=torch.float32, device="cuda")
    print("full-size prefill: attention launch", flush=True)
    W.wsvd_prefill_attn(L.ctx, d, as_dtype_dev(q32, "bf16"), T, 0, as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16"),
                        L.cache, T, out)
    torch.cuda.synchronize()
    assert W.wsvd_check(L.ctx) == 0
    assert bool(torch.isfinite(out).all())
    toks = [(b, int(kv), int(i)) for b in seqs for kv in rng.integers(0, sp.n_kv_heads, 3)
            for i in (0, 31, 32, 1000, T - 33, T - 1)]
    ref = O.causal_attn_reconstructed(oc, q32, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale, tokens=toks)
    got = np.full(q32.shape, np.nan)
    for t in toks:
        got[t] = out[t].cpu().numpy()
    check_out(got, ref, "i8", f"full-size prompt attention, {len(toks)} sampled (sequence, head, token) triples")
    L.close()


def test_prefill_all_sequences_capacity_of_some():
    """seq_index = -1 with sequences of different lengths: those whose prompt does not fit are left full and reported,
    the rows that fit are stored for all of them, the others advance by the whole prompt."""
    c = build_case("c3_small", extra_cap=70)
    sp = c.sp
    c.cache.seq_lens[:] = [333, 400, 250]         # (rows past the built context hold the cache's initial contents)
    L = layer_for(c); L.upload(c.cache)
    n = 100
    X = np.stack([WI.bf16_exact(WI.hidden_states(sp, n, 1.0, which="ctx", sub=90 + b)) for b in range(sp.batch)])
    xd = as_dtype_dev(X.reshape(sp.batch * n, -1), "bf16")
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    starts = c.cache.seq_lens.copy()
    room = L.t_cap - starts
    assert (room < n).any() and (room >= n).any(), "the case needs both kinds of sequences"
    over = [O.latent_prefill(c.cache, b, X[b].astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
            for b in range(sp.batch)]
    assert over == [bool(r < n) for r in room]
    W.wsvd_prefill_append(L.ctx, L.desc, xd, None, n, -1, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == W.E_CAPACITY
    want = np.minimum(starts + n, L.t_cap)
    assert (L.seq_lens.cpu().numpy() == want).all() and (c.cache.seq_lens == want).all()
    for b in range(sp.batch):
        _compare_rows(L, c.cache, b, int(starts[b]), int(want[b] - starts[b]), "i8", _latents64(X[b], c.AK), _latents64(X[b], c.AV))
    L.close()


def _check_i4_rows(L, plane, b, t0, n, values64, what):
    """int4 rows [t0, t0 + n) of sequence b written by the GPU from fp32 sums, against the asymmetric rule applied to the
    oracle's fp64 latents values64 [Hkv, n, r].  A row's scale / zero point may differ from the fp64 rule's only where
    (hi - lo) / 15 sits within 1e-5 (relative) of the midpoint between two fp16 values, or -lo / s within 1e-3 of a .5
    rounding boundary; its codes are then checked against the rule applied with the GPU's own scale and zero point.  A
    code may differ by one step only where value / scale lies within 1e-3 of .5.  Returns the number of accepted flips."""
    gc, gs, gz = L.download(plane, t0, n)
    codes = O.unpack_int4(gc[b].reshape(-1, gc.shape[-1])).reshape(gc.shape[1], n, -1).astype(np.int64)     # [Hkv, n, r]
    gs = gs[b].astype(np.float64); gz = gz[b].astype(np.float64)
    v = np.asarray(values64, np.float64)
    lo = np.minimum(v.min(-1), 0.0); hi = np.maximum(v.max(-1), 0.0)
    flat = hi == lo
    s_exact = np.where(flat, 1.0, (hi - lo) / 15.0)
    s_ref = np.where(flat, 1.0, s_exact.astype(np.float32).astype(np.float16).astype(np.float64))
    flips = 0
    ds = gs != s_ref
    if ds.any():
        # the two fp16 neighbours of the exact value and their midpoint
        f16 = s_exact[ds].astype(np.float16)
        nb = np.where(f16.astype(np.float64) < s_exact[ds], np.nextafter(f16, np.float16(np.inf)), np.nextafter(f16, np.float16(-np.inf)))
        mid = 0.5 * (f16.astype(np.float64) + nb.astype(np.float64))
        assert (np.abs(s_exact[ds] - mid) <= 1e-5 * s_exact[ds]).all(), f"{what}: a scale differs away from an fp16 rounding boundary"
        assert (np.abs(gs[ds] - s_ref[ds]) <= np.abs(nb.astype(np.float64) - f16.astype(np.float64)) * 1.001).all()
        flips += int(ds.sum())
    z_exact = np.where(flat, 0.0, -lo / gs)
    z_ref = np.clip(np.rint(z_exact), 0, 15)
    dz = gz != z_ref
    if dz.any():
        frac = z_exact[dz] - np.floor(z_exact[dz])
        assert (np.abs(gz[dz] - z_ref[dz]) == 1).all() and (np.abs(frac - 0.5) < 1e-3).all(), f"{what}: a zero point differs away from a rounding boundary"
        flips += int(dz.sum())
    x = v / gs[..., None]
    want = np.clip(np.clip(np.rint(x), -64, 64) + gz[..., None], 0, 15).astype(np.int64)
    bad = codes != want
    if bad.any():
        frac = x[bad] - np.floor(x[bad])
        assert (np.abs(codes[bad] - want[bad]) == 1).all() and (np.abs(frac - 0.5) < 1e-3).all(), \
            f"{what}: {int(bad.sum())} codes differ away from a rounding boundary"
        flips += int(bad.sum())
    assert flips <= max(3, codes.size // 300), f"{what}: {flips} boundary flips in {codes.size} codes is too many to be rounding"
    return flips


@pytest.mark.parametrize("all_seqs", [False, True], ids=["one-sequence", "all-sequences"])
def test_prefill_int4_tiled(all_seqs):
    """int4 latents through the tiled projection: a value byte holds two consecutive rows, so both rows of a byte are
    written from one place; the target sequences stand at even lengths (0, or an even number of uploaded rows)."""
    c = build_case("c4_small", extra_cap=300, batch=4, context=300, ragged=(100, 300))
    sp = c.sp
    lens = (c.cache.seq_lens // 2 * 2).astype(np.int32)
    lens[1] = 0                                             # a fresh sequence
    c.cache.seq_lens[:] = lens
    assert c.t_cap >= 300 + 151 + 1
    L = layer_for(c); L.upload(c.cache)
    n = 151 if not all_seqs else 70                        # odd counts: the last row of the block has no partner yet
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    if all_seqs:
        X = np.stack([WI.bf16_exact(WI.hidden_states(sp, n, 1.0, which="ctx", sub=60 + b)) for b in range(sp.batch)])
        W.wsvd_prefill_append(L.ctx, L.desc, as_dtype_dev(X.reshape(sp.batch * n, -1), "bf16"), None, n, -1, AKd, AVd, L.cache)
        targets = list(range(sp.batch))
    else:
        b = 2
        X = np.zeros((sp.batch, n, sp.d_model), np.float32)
        X[b] = WI.bf16_exact(WI.hidden_states(sp, n, 1.0, which="ctx", sub=77))
        W.wsvd_prefill_append(L.ctx, L.desc, as_dtype_dev(X[b], "bf16"), None, n, b, AKd, AVd, L.cache)
        targets = [b]
    assert W.wsvd_check(L.ctx) == 0
    got_lens = L.seq_lens.cpu().numpy()
    for b in range(sp.batch):
        assert got_lens[b] == lens[b] + (n if b in targets else 0)
    total = 0
    for b in targets:
        for plane, A in ((0, c.AK), (1, c.AV)):
            total += _check_i4_rows(L, plane, b, int(lens[b]), n, _latents64(X[b], A), f"int4 prefill seq {b} plane {plane}")
    print(f"int4 prefill ({'all' if all_seqs else 'one'}): {total} boundary flips accepted", flush=True)
    # the rows that were there before are untouched (the first new row shares no byte with them: it is an even row)
    for b in targets:
        if lens[b]:
            for plane, oc in ((0, c.cache.k), (1, c.cache.v)):
                gc, _, _ = L.download(plane, 0, int(lens[b]))
                assert (gc[b] == oc[b, :, : int(lens[b])]).all()
    # one more token on top goes through the ordinary append (odd row: read-modify-write of the shared byte), then the
    # attention over everything matches the oracle run on the same hidden states
    for b in targets:
        assert not O.latent_prefill(c.cache, b, X[b].astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    x1 = WI.bf16_exact(c.x_new[0])
    O.latent_append(c.cache, x1.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    assert L.append(as_dtype_dev(x1, "bf16"), None, AKd, AVd) == 0
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    got = L.attend(qd, qs, as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16"), int(c.cache.seq_lens.max()))
    ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    check_out(got, ref, "i4", "attention over an int4 cache built by the tiled prefill")
    # a sequence that stands at an odd length is left alone and reported
    odd = int(np.nonzero(L.seq_lens.cpu().numpy() % 2 == 1)[0][0])
    before = int(L.seq_lens[odd])
    W.wsvd_prefill_append(L.ctx, L.desc, as_dtype_dev(X[targets[0]][:8], "bf16"), None, 8, odd, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == W.E_SHAPE and int(L.seq_lens[odd]) == before
    L.close()
