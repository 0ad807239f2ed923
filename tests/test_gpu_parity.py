"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle on identical seeded inputs.

Bars (from the benchmark spec): quantise / pack / index work bit-exact; fp32 path <= 1e-5 relative
(max abs error over max |reference|); bf16 and integer-latent paths <= 2e-2 max-abs; <= 1e-3 relative L2
everywhere.  Attention tests read caches written by the ORACLE (uploaded through wsvd_cache_import), so a
quantiser flip on the GPU cannot leak into them; the append tests compare the GPU-written cache with the
oracle's, allowing a differing code only where fp32-vs-fp64 summation can legitimately flip a rounding.
"""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
import wsvd_inputs as WI
from cases import build_case, round_up
from harness import DeviceLayer, as_dtype_dev, dev, err_stats, q_to_device

pytestmark = pytest.mark.gpu

TOL = {"f32": dict(rel_max=1e-5, rel_l2=1e-5), "bf16": dict(abs_max=2e-2, rel_l2=1e-3),
       "i8": dict(abs_max=2e-2, rel_l2=1e-3), "i4": dict(abs_max=2e-2, rel_l2=1e-3),
       # the rotary variant carries N as an fp16 pair (22 bits): far inside the int8 bar.  The tighter figures are there
       # to catch a lost or mismatched low term (one entry off by an fp16 step gave 1.8e-4 / 1.6e-5); observed
       # 2e-5 .. 4e-5 max abs, 2e-6 .. 4e-6 rel L2
       "rope": dict(abs_max=1e-4, rel_l2=1e-5)}


def check_out(got, ref, dtype, what=""):
    mask = ~np.isnan(ref)
    assert np.isfinite(got[mask]).all(), f"{what}: non-finite output"
    a, r, l2 = err_stats(got[mask], ref[mask])
    t = TOL[dtype]
    print(f"{what}: max_abs={a:.3e} rel_max={r:.3e} rel_l2={l2:.3e}", flush=True)
    if "abs_max" in t:
        assert a <= t["abs_max"], f"{what}: max abs {a} > {t['abs_max']}"
    if "rel_max" in t:
        assert r <= t["rel_max"], f"{what}: rel max {r} > {t['rel_max']}"
    assert l2 <= t["rel_l2"], f"{what}: rel L2 {l2} > {t['rel_l2']}"


def layer_for(c, t_cap=None, min_chunk=256):
    sp = c.sp
    return DeviceLayer(sp.batch, sp.n_q_heads, sp.n_kv_heads, sp.d_head, sp.d_model, sp.rank, t_cap or c.t_cap,
                       sp.latent_dtype, sp.factor_dtype, "f32" if sp.factor_dtype == "f32" else "bf16", sp.q_dtype,
                       c.sm_scale, min_chunk=min_chunk)


def run_attend(c, L, step=0, heads=None, max_len=None):
    sp = c.sp
    qd, qs, q64 = q_to_device(c.q32[step], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, sp.factor_dtype), as_dtype_dev(c.BV, sp.factor_dtype)
    got = L.attend(qd, qs, BKd, BVd, int(max_len if max_len is not None else c.cache.seq_lens.max()))
    ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale, heads=heads)
    return got, ref


# ------------------------------------------------------------------------------------------ quantiser
def _tricky_rows(rng, n, r):
    c = (rng.standard_normal((n, r)) * np.exp(rng.standard_normal((n, 1)) * 3)).astype(np.float32)
    c[0] = 0
    c[1] = np.float32(1e-9) * c[1]                       # fp16-subnormal scale
    c[2] = np.float32(3e6) * np.sign(c[2] + 0.1)         # fp16 scale overflow -> 65504
    c[3, :] = 0; c[3, 5] = 127.0                         # scale exactly 1: ties on the codes
    c[3, :5] = [0.5, 1.5, 2.5, -0.5, -1.5]
    c[4] = np.abs(c[4]); c[5] = -np.abs(c[5])            # one-sided rows (int4 zero point 0 / 15)
    c[6] = 1e-30                                         # scale underflows to the 2^-24 guard
    c[7, :] = np.float32(2.0 ** -20)
    return c


@pytest.mark.parametrize("dtype,r", [("i8", 32), ("i8", 64), ("i4", 32)])
def test_quantize_rows_bit_exact(dtype, r):
    rng = np.random.default_rng(100 + r)
    n = 5000
    c = _tricky_rows(rng, n, r)
    L = DeviceLayer(1, 1, 1, 128, 512, r, 64, dtype, "bf16", "bf16", "i8")
    cd = dev(c)
    codes = torch.zeros((n, r if dtype == "i8" else r // 2), dtype=torch.uint8, device="cuda")
    meta = torch.zeros((n, 1 if dtype == "i8" else 2), dtype=torch.int16, device="cuda")
    W.wsvd_quantize_rows(L.ctx, L.desc, cd, n, codes, meta)
    assert W.wsvd_check(L.ctx) == 0
    gc = codes.cpu().numpy(); gm = meta.cpu().numpy().view(np.uint16)
    if dtype == "i8":
        oc, os_ = O.quantize_int8_rows(c)
        assert (gm[:, 0] == os_.view(np.uint16)).all(), "scale bits differ"
        assert (gc.view(np.int8) == oc).all(), "codes differ"
    else:
        oc, os_, oz = O.quantize_int4_rows(c)
        assert (gm[:, 0] == os_.view(np.uint16)).all() and (gm[:, 1] == oz.view(np.uint16)).all(), "scale / zero bits differ"
        assert (gc == oc).all(), "packed codes differ"
    L.close()


@pytest.mark.parametrize("rows,cols,dt", [(37, 3584, "f32"), (5, 16384, "f32"), (3, 16388, "f32"), (4, 4098, "f32"),
                                          (2, 40, "f32"), (6, 1792, "bf16"), (3, 32768, "bf16"), (2, 36, "bf16")])
def test_quantize_act_i8_bit_exact(rows, cols, dt):
    """Both activation-quantiser kernels (rows kept in registers; the strided fallback for long or odd rows)."""
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((rows, cols)) * np.exp(rng.standard_normal((rows, 1)))).astype(np.float32)
    x[0] = 0
    if dt == "bf16":
        x = WI.bf16_exact(x)
    L = DeviceLayer(1, 1, 1, 128, 512, 32, 64, "i8", "bf16", "bf16", "i8")
    codes = torch.zeros((rows, cols), dtype=torch.int8, device="cuda"); sc = torch.zeros(rows, dtype=torch.int16, device="cuda")
    W.wsvd_quantize_act_i8(L.ctx, as_dtype_dev(x, dt), dt, rows, cols, codes, sc)
    assert W.wsvd_check(L.ctx) == 0
    oc, os_ = O.quantize_act_i8(x)
    assert (sc.cpu().numpy().view(np.uint16) == os_.view(np.uint16)).all()
    assert (codes.cpu().numpy() == oc).all()
    L.close()


# ------------------------------------------------------------------------------------------ layout copies
@pytest.mark.parametrize("dtype,r", [("f32", 16), ("bf16", 32), ("i8", 32), ("i8", 64), ("i4", 32)])
def test_cache_import_export_round_trip(dtype, r):
    rng = np.random.default_rng(5)
    B, Hkv, t_cap = 2, 3, 192
    oc = O.LatentCache(B, Hkv, t_cap, r, dtype)
    for b in range(B):
        oc.store_rows("k", b, 0, rng.standard_normal((Hkv, t_cap, r)) * 3)
        oc.store_rows("v", b, 0, rng.standard_normal((Hkv, t_cap, r)) * 3)
    fd = "f32" if dtype == "f32" else "bf16"
    L = DeviceLayer(B, Hkv, Hkv, 128 if r > 16 else 64, 512, r, t_cap, dtype, fd, fd, fd if dtype in ("f32", "bf16") else "i8")
    L.upload(oc, n_rows=t_cap, keep_poison=False)      # all rows as they are (the lengths stay 0: only the copies are tested)
    for plane, codes, scale, zero in ((0, oc.k, oc.k_scale, oc.k_zero), (1, oc.v, oc.v_scale, oc.v_zero)):
        for (t0, n) in ((0, t_cap), (5, 61), (64, 1), (33, 2)):
            gc, gs, gz = L.download(plane, t0, n)
            assert (gc.reshape(codes[:, :, t0:t0 + n].shape) == codes[:, :, t0:t0 + n]).all(), (plane, t0, n)
            if scale is not None:
                assert (gs.view(np.uint16) == scale[:, :, t0:t0 + n].view(np.uint16)).all()
            if zero is not None:
                assert (gz.view(np.uint16) == zero[:, :, t0:t0 + n].view(np.uint16)).all()
    # a partial import (odd start, odd length) must leave every other row untouched
    oc2 = O.LatentCache(B, Hkv, t_cap, r, dtype)
    for b in range(B):
        oc2.store_rows("k", b, 0, rng.standard_normal((Hkv, t_cap, r))); oc2.store_rows("v", b, 0, rng.standard_normal((Hkv, t_cap, r)))
    t0, n = 67, 5
    for plane, src in ((0, oc2.k), (1, oc2.v)):
        meta = None
        if dtype == "i8":
            meta = dev((oc2.k_scale if plane == 0 else oc2.v_scale)[:, :, t0:t0 + n].view(np.uint16))
        if dtype == "i4":
            s = (oc2.k_scale if plane == 0 else oc2.v_scale)[:, :, t0:t0 + n].view(np.uint16)
            z = (oc2.k_zero if plane == 0 else oc2.v_zero)[:, :, t0:t0 + n].view(np.uint16)
            meta = dev(np.stack([s, z], axis=-1))
        W.wsvd_cache_import(L.ctx, L.desc, plane, dev(src[:, :, t0:t0 + n]), meta, t0, n, L.cache)
        gc, _, _ = L.download(plane, 0, t_cap)
        want = (oc.k if plane == 0 else oc.v).copy(); want[:, :, t0:t0 + n] = src[:, :, t0:t0 + n]
        assert (gc.reshape(want.shape) == want).all()
    L.close()


# ------------------------------------------------------------------------------------------ attention, small shapes
SMALL = [
    # name, overrides
    ("c1", dict(batch=2, context=100)),
    ("c1", dict()),
    ("c2_small", dict()),
    ("c3_small", dict()),
    ("c3_small", dict(n_q_heads=8, n_kv_heads=4)),           # G = 2
    ("c3_small", dict(n_q_heads=12, n_kv_heads=4)),          # G = 3
    ("c3_small", dict(n_q_heads=16, n_kv_heads=4)),          # G = 4
    ("c3_small", dict(rank=64, context=700)),                # rank 64, several chunks
    ("c3_small", dict(q_dtype="f32")),
    ("c4_small", dict()),
    ("c4_small", dict(n_q_heads=8, n_kv_heads=4, q_dtype="bf16")),
    ("c5_small", dict(n_q_heads=8, n_kv_heads=2)),           # rank 64, G = 4 (paired-block kernel)
    ("c5_small", dict()),                                    # rank 64, G = 7 (one-block-per-MFMA kernel)
    ("c5_small", dict(n_q_heads=10)),                        # G = 5
    ("c5_small", dict(n_q_heads=12)),                        # G = 6
    ("c5_small", dict(n_q_heads=16, d_head=64)),             # G = 8, d_head 64
    ("c5_small", dict(context=2000)),                        # G = 7 over several context chunks
    ("c3_small", dict(n_q_heads=28, n_kv_heads=4)),          # G = 7, rank 32, int8 query
    ("c2_small", dict(n_q_heads=12)),                        # bf16 latents, G = 3
    ("c2_small", dict(n_q_heads=28)),                        # bf16 latents, G = 7
    ("c2_small", dict(n_q_heads=32, rank=64)),               # bf16 latents, G = 8, rank 64
    ("c1", dict(n_q_heads=40, n_kv_heads=8)),                # fp32 latents, G = 5
    ("c4_small", dict(n_q_heads=28, n_kv_heads=4)),          # int4 latents, G = 7: two launches over head groups (4 + 3)
    ("c4_small", dict(n_q_heads=20, n_kv_heads=4, q_dtype="f32", context=2000, ragged=())),   # int4, G = 5 (4 + 1), several chunks
]


@pytest.mark.parametrize("name,over", SMALL, ids=[f"{n}-{'-'.join(f'{k}{v}' for k, v in o.items())}" for n, o in SMALL])
def test_attention_small(name, over):
    c = build_case(name, **over)
    L = layer_for(c)
    L.upload(c.cache)
    got, ref = run_attend(c, L)
    check_out(got, ref, c.sp.latent_dtype, f"{name}{over}")
    L.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i8", "i4", "i8-gqa7"])
def test_attention_edge_lengths(dtype):
    """Empty sequences, a single row, lengths around the 32-row block, the 64-row tile and the chunk boundary, one
    sequence at capacity."""
    name = {"f32": "c1", "bf16": "c2_small", "i8": "c3_small", "i4": "c4_small", "i8-gqa7": "c5_small"}[dtype]
    dtype = dtype.split("-")[0]
    lens = [0, 1, 2, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 255, 256, 257, 511, 512, 640]
    c = build_case(name, batch=len(lens), context=640, ragged=(), extra_cap=0, steps=1)
    for b, n in enumerate(lens):
        c.cache.seq_lens[b] = n
    L = layer_for(c)
    L.upload(c.cache)
    got, ref = run_attend(c, L)
    assert (got[0] == 0).all(), "empty sequence must give zeros"
    check_out(got, ref, dtype, f"edge-{dtype}")
    # n = 1: the output is that row's V exactly (softmax weight 1)
    L.close()


@pytest.mark.parametrize("dtype", ["f32", "i8", "i4", "i8-gqa7"])
def test_attention_independent_of_split_count(dtype):
    """The result may depend on the number of context splits only through fp32 rounding."""
    name = {"f32": "c1", "i8": "c3_small", "i4": "c4_small", "i8-gqa7": "c5_small"}[dtype]
    dtype = dtype.split("-")[0]
    c = build_case(name, batch=2, context=1500, ragged=())
    L = layer_for(c)
    L.upload(c.cache)
    outs = []
    W.wsvd_ctx_set_option(L.ctx, "min_chunk", 0)      # the library's own policy (the harness pins 256-row chunks)
    got, ref = run_attend(c, L)             # default policy: one large workgroup per (sequence, kv head)
    check_out(got, ref, dtype, "splits default policy")
    outs.append(got)
    try:
        W.wsvd_ctx_set_option(L.ctx, "max_threads", 256)
        for mc in (2048, 1024, 512, 256):   # 1, 2, 3 and 6 context chunks per (sequence, kv head)
            W.wsvd_ctx_set_option(L.ctx, "min_chunk", mc)
            got, ref = run_attend(c, L)
            check_out(got, ref, dtype, f"splits min_chunk={mc}")
            outs.append(got)
        # the settings belong to L's context: a second context on the same cache still launches the default policy
        other = W.wsvd_create(0)
        ws2 = torch.empty(W.wsvd_workspace_bytes(L.desc), dtype=torch.uint8, device="cuda")
        W.wsvd_set_workspace(other, ws2)
        qd, qs, _ = q_to_device(c.q32[0], c.sp.q_dtype)
        fd = c.sp.factor_dtype
        out2 = torch.full_like(L.out, float("nan"))
        W.wsvd_decode_attn(other, L.desc, qd, qs, as_dtype_dev(c.BK, fd), as_dtype_dev(c.BV, fd), L.cache, int(c.cache.seq_lens.max()), out2)
        assert W.wsvd_check(other) == 0
        assert (out2.cpu().numpy().astype(np.float64) == outs[0]).all(), "a context's settings leaked into another context"
        W.wsvd_destroy(other)
    finally:
        W.wsvd_ctx_set_option(L.ctx, "min_chunk", 256)
        W.wsvd_ctx_set_option(L.ctx, "max_threads", 0)
    # each variant sits 2e-5 .. 6e-5 (max abs; 4e-6 .. 7e-6 rel L2) from the oracle through its own order of fp32 sums and
    # its own reference maxima for the probabilities' limbs: two variants differ by at most the sum of two such errors
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() <= 2.5e-5 * np.abs(outs[0]).max()
    # repeatability: same launch twice gives identical bits (fixed merge order)
    g1, _ = run_attend(c, L); g2, _ = run_attend(c, L)
    assert (g1 == g2).all()
    assert any((o != outs[0]).any() for o in outs[1:]), "split count had no effect: the option is not reaching the launch"
    L.close()


def test_attention_reports_a_too_small_length_bound():
    """max_seq_len is the caller's promise; a longer sequence must be reported, not silently truncated."""
    c = build_case("c3_small", context=900)
    L = layer_for(c); L.upload(c.cache)
    qd, qs, q64 = q_to_device(c.q32[0], c.sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    W.wsvd_decode_attn(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, 200, L.out)      # 900 rows, bound 200
    assert W.wsvd_check(L.ctx) == W.E_SHAPE
    W.wsvd_decode_attn(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, 900, L.out)      # honest bound: clean again
    assert W.wsvd_check(L.ctx) == 0
    L.close()


@pytest.mark.parametrize("name,over", [("c3_small", dict(context=2000, batch=4)), ("c5_small", dict(context=2000)),
                                       ("c4_small", dict(batch=6, context=1800, ragged=(900, 1800)))],
                         ids=["i8", "i8-gqa7", "i4-ragged"])
def test_cross_workgroup_handoffs_are_repeatable(name, over):
    """Split merges and the append's slice hand-off go through tickets and write-through stores; a hand-off that is
    not properly ordered shows up as a result that changes from launch to launch.  40 launches each, bit-identical."""
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    n_max = int(c.cache.seq_lens.max())
    try:
        W.wsvd_ctx_set_option(L.ctx, "min_chunk", 256)
        W.wsvd_ctx_set_option(L.ctx, "max_threads", 256)          # many small chunks per sequence
        first = None
        for it in range(40):
            got = L.attend(qd, qs, BKd, BVd, n_max)
            if first is None:
                first = got
                ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
                check_out(got, ref, sp.latent_dtype, f"repeatable {name}")
            assert (got == first).all(), f"launch {it} differs from launch 0"
    finally:
        W.wsvd_ctx_set_option(L.ctx, "max_threads", 0)
    if sp.n_q_heads // sp.n_kv_heads > 4:
        L.close()
        return
    # the append, 30 times from the same state: identical rows every time
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    x = as_dtype_dev(WI.bf16_exact(c.x_new[0]), "bf16")
    lens = c.cache.seq_lens.copy()
    rows0 = None
    for it in range(30):
        L.seq_lens.copy_(torch.from_numpy(lens.astype(np.int32)))
        assert L.append(x, None, AKd, AVd) == 0
        rows = []
        for plane in (0, 1):
            gc, gs, gz = L.download(plane, int(lens.min()), int(lens.max() - lens.min()) + 1)
            rows += [gc.copy(), gs.copy()] + ([gz.copy()] if gz is not None else [])
        if rows0 is None:
            rows0 = rows
        # bit patterns, not values: rows past a shorter sequence's end hold NaN metadata
        assert all(a.tobytes() == b.tobytes() for a, b in zip(rows, rows0)), f"append {it} differs from append 0"
    L.close()


@pytest.mark.parametrize("name", ["c1", "c2_small", "c3_small", "c4_small", "c5_small"], ids=["f32", "bf16", "i8", "i4", "i8r64g7"])
def test_append_then_attend_from_never_written_cache(name):
    """Nothing is uploaded: the planes hold the poison pattern (codes 0xA5, metadata and float latents NaN bits) that
    stands for memory the append never wrote, the lengths start at 0, and every row comes from wsvd_latent_append.
    The attention is checked at lengths inside the first 32-row block, across the 64-row tile edge and past it: a kernel
    that lets a never-written row of its last tile reach the result (a NaN scale or zero point times a zero weight)
    returns NaN here."""
    steps = 70
    c = build_case(name, batch=3, steps=steps)
    sp = c.sp
    oc = O.LatentCache(sp.batch, sp.n_kv_heads, c.t_cap, sp.rank, sp.latent_dtype)
    L = layer_for(c)
    fd = sp.factor_dtype
    AKd, AVd = L.pack_A(c.AK, fd), L.pack_A(c.AV, fd)
    BKd, BVd = as_dtype_dev(c.BK, fd), as_dtype_dev(c.BV, fd)
    AK64, AV64, BK64, BV64 = (a.astype(np.float64) for a in (c.AK, c.AV, c.BK, c.BV))
    for step in range(steps):
        x = c.x_new[step] if fd == "f32" else WI.bf16_exact(c.x_new[step])
        assert not O.latent_append(oc, x.astype(np.float64), AK64, AV64).any()
        assert L.append(as_dtype_dev(x, fd), None, AKd, AVd) == 0
        if step + 1 in (1, 2, 31, 33, 63, 64, 65, 70):
            qd, qs, q64 = q_to_device(c.q32[step], sp.q_dtype)
            got = L.attend(qd, qs, BKd, BVd, step + 1)
            ref = O.decode_attn_reconstructed(oc, q64, BK64, BV64, c.sm_scale)
            check_out(got, ref, sp.latent_dtype, f"never-written cache {name}, {step + 1} rows")
    assert (L.seq_lens.cpu().numpy() == steps).all()
    L.close()


@pytest.mark.parametrize("name,over", [("c4_small", dict()), ("c3_small", dict()), ("c5_small", dict()),
                                       ("c4_small", dict(n_q_heads=16, n_kv_heads=4))], ids=["i4", "i8", "i8r64g7", "i4g4"])
def test_rows_past_the_end_hold_nan_metadata(name, over):
    """Regression: the last tile of a sequence whose length is not a multiple of 64 ends in rows that were never
    written; their scale and zero point are fp16 NaN here, their codes 0xA5.  The output must be finite and right."""
    c = build_case(name, batch=4, context=300, ragged=(), extra_cap=64, **over)
    for b, n in enumerate((1, 37, 65, 299)):
        c.cache.seq_lens[b] = n
    L = layer_for(c); L.upload(c.cache)
    meta = L.k_meta.cpu().numpy()
    assert (meta[-64:] == 0xFF).all(), "the case needs poisoned rows behind the last sequence"
    got, ref = run_attend(c, L)
    check_out(got, ref, c.sp.latent_dtype, f"NaN metadata past the end, {name}{over}")
    L.close()


def test_large_scores_stay_finite():
    c = build_case("c3_small", q_dtype="f32")
    c.q32 = c.q32 * 200.0
    L = layer_for(c); L.upload(c.cache)
    got, ref = run_attend(c, L)
    check_out(got, ref, "i8", "large scores")
    L.close()


# ------------------------------------------------------------------------------------------ append
def _append_compare(L, oc, c64K, c64V, t_rows, dtype, only=None):
    """Compare GPU-written rows with the oracle's; c64K/V [B,Hkv,r] are the oracle's fp64 latents."""
    flips = 0
    for plane, ocodes, oscale, ozero, c64 in ((0, oc.k, oc.k_scale, oc.k_zero, c64K), (1, oc.v, oc.v_scale, oc.v_zero, c64V)):
        for b in (range(oc.B) if only is None else only):
            t = int(t_rows[b])
            gc, gs, gz = L.download(plane, t, 1)
            gc = gc[b, :, 0]; want = ocodes[b, :, t]
            cc = c64[b]
            if dtype == "f32":
                scale = np.abs(cc).max()
                assert np.abs(gc.astype(np.float64) - cc).max() <= 1e-5 * scale
            elif dtype == "bf16":
                gv = O.f64_from_bf16_bits(gc)
                ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(cc), 1e-300))) - 7)
                assert (np.abs(gv - cc) <= 0.5 * ulp + 1e-5 * np.abs(cc).max()).all()
                flips += int((gc != want).sum())
            else:
                gsb = gs[b, :, 0]; osb = oscale[b, :, t]
                for h in range(oc.Hkv):
                    assert gsb[h] == osb[h], f"scale differs b={b} h={h}: {gsb[h]} vs {osb[h]} (abs-max boundary cases are not expected in this data)"
                    s = float(gsb[h])
                    if dtype == "i8":
                        g = gc[h].astype(np.int64); o_ = want[h].astype(np.int64)
                    else:
                        assert gz[b, h, 0] == ozero[b, h, t]
                        g = O.unpack_int4(gc[h]).astype(np.int64); o_ = O.unpack_int4(want[h]).astype(np.int64)
                    bad = np.nonzero(g != o_)[0]
                    for j in bad:
                        frac = cc[h, j] / s - np.floor(cc[h, j] / s)
                        assert abs(int(g[j]) - int(o_[j])) == 1 and abs(frac - 0.5) < 1e-3, \
                            f"code differs away from a rounding boundary: b={b} h={h} j={j} gpu={g[j]} oracle={o_[j]} c/s={cc[h, j] / s}"
                    flips += len(bad)
    return flips


@pytest.mark.parametrize("name,over", [("c1", dict(batch=3, context=70)), ("c2_small", dict()), ("c3_small", dict()),
                                       ("c4_small", dict()), ("c3_small", dict(rank=64, batch=11)),
                                       ("c3_small", dict(batch=40, context=130)), ("c4_small", dict(batch=70, context=200, ragged=(1, 200))),
                                       ("c3_small", dict(batch=33, rank=64, context=100))],
                         ids=["f32", "bf16", "i8", "i4", "i8r64b11", "i8b40", "i4b70", "i8r64b33"])
def test_append_matches_oracle(name, over):
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c)
    L.upload(c.cache)
    xdt = "f32" if sp.factor_dtype == "f32" else "bf16"
    AKd, AVd = L.pack_A(c.AK, sp.factor_dtype), L.pack_A(c.AV, sp.factor_dtype)
    total_flips = 0
    for step in range(min(sp.steps, 3) if sp.steps > 1 else 2):
        x = c.x_new[step % c.x_new.shape[0]]
        if xdt == "bf16":
            x = WI.bf16_exact(x)
        before = c.cache.seq_lens.copy()
        x64 = x.astype(np.float64)
        cK = O.project_latents(x64, c.AK.astype(np.float64)); cV = O.project_latents(x64, c.AV.astype(np.float64))
        ov = O.latent_append(c.cache, x64, c.AK.astype(np.float64), c.AV.astype(np.float64))
        assert not ov.any()
        st = L.append(as_dtype_dev(x, xdt), None, AKd, AVd)
        assert st == 0, W.status_str(st)
        assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all(), "seq_lens not advanced by exactly one"
        total_flips += _append_compare(L, c.cache, cK, cV, before, sp.latent_dtype)
        # continue from the oracle's cache so that later steps compare like with like
        L.upload(c.cache)
    print(f"append {name}: boundary flips accepted = {total_flips}", flush=True)
    n_codes = 2 * sp.batch * sp.n_kv_heads * sp.rank * 3
    assert total_flips <= max(2, n_codes // 500), "too many rounding flips to be boundary cases"
    L.close()


@pytest.mark.parametrize("name", ["c3_small", "c4_small"], ids=["i8", "i4"])
def test_append_quantised_partly_filled_groups(name):
    """The lanes of a wave quantise several rows side by side.  Groups that do not fill a wave: three sequences with the
    middle one at capacity (its lanes take part in the reductions and store nothing; reported, left untouched), then a
    single sequence."""
    c = build_case(name, batch=3)
    sp = c.sp
    AK64, AV64 = c.AK.astype(np.float64), c.AV.astype(np.float64)
    L = layer_for(c)
    c.cache.seq_lens[:] = [5, c.t_cap, 0]
    L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    held = [L.download(pl, 0, c.t_cap) for pl in (0, 1)]
    x = WI.bf16_exact(c.x_new[0]); x64 = x.astype(np.float64)
    cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
    before = c.cache.seq_lens.copy()
    full = O.latent_append(c.cache, x64, AK64, AV64)
    assert full.tolist() == [False, True, False]
    st = L.append(as_dtype_dev(x, "bf16"), None, AKd, AVd)
    assert st == 5, "capacity overflow must be reported by wsvd_check"
    assert L.seq_lens.cpu().numpy().tolist() == [6, c.t_cap, 1]
    flips = _append_compare(L, c.cache, cK, cV, before, sp.latent_dtype, only=(0, 2))
    for pl in (0, 1):
        now = L.download(pl, 0, c.t_cap)
        for a, b in zip(held[pl], now):
            if a is not None:
                assert a[1].tobytes() == b[1].tobytes(), "a sequence at capacity must not be modified"
    L.close()
    c = build_case(name, batch=1)
    AK64, AV64 = c.AK.astype(np.float64), c.AV.astype(np.float64)
    L = layer_for(c); L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    x = WI.bf16_exact(c.x_new[0]); x64 = x.astype(np.float64)
    cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
    before = c.cache.seq_lens.copy()
    assert not O.latent_append(c.cache, x64, AK64, AV64).any()
    st = L.append(as_dtype_dev(x, "bf16"), None, AKd, AVd)
    assert st == 0, W.status_str(st)
    assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    flips += _append_compare(L, c.cache, cK, cV, before, sp.latent_dtype)
    assert flips <= 2
    L.close()


@pytest.mark.parametrize("name", ["c3_small", "c4_small"], ids=["i8", "i4"])
def test_append_int8_hidden_states(name):
    """x given as int8 codes with one fp16 scale per token (the activation format of Section 4.2): the latents are those
    of the dequantised hidden state.  Decode append (two steps), then a prefill call of a few tokens of one sequence, then
    attention over everything against the oracle."""
    c = build_case(name)
    sp = c.sp
    L = DeviceLayer(sp.batch, sp.n_q_heads, sp.n_kv_heads, sp.d_head, sp.d_model, sp.rank, c.t_cap, sp.latent_dtype, "bf16", "i8",
                    sp.q_dtype, c.sm_scale)
    L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    AK64, AV64 = c.AK.astype(np.float64), c.AV.astype(np.float64)
    flips = 0
    for step in range(2):
        codes, s = O.quantize_act_i8(c.x_new[step % c.x_new.shape[0]])
        x64 = codes.astype(np.float64) * s.astype(np.float64)[:, None]
        before = c.cache.seq_lens.copy()
        cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
        assert not O.latent_append(c.cache, x64, AK64, AV64).any()
        assert L.append(dev(codes), dev(s.view(np.uint16)), AKd, AVd) == 0
        assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
        flips += _append_compare(L, c.cache, cK, cV, before, sp.latent_dtype)
        L.upload(c.cache)
    assert flips <= 2
    if sp.latent_dtype == "i8":        # (int4 latents take the tiled prefill, which wants bf16 hidden states)
        n_tok, b = sp.batch, 1             # (the layer's workspace is sized for `batch` rows of x)
        X = WI.hidden_states(sp, n_tok, 1.0, which="new", sub=77)
        codes, s = O.quantize_act_i8(X)
        X64 = codes.astype(np.float64) * s.astype(np.float64)[:, None]
        n0 = int(c.cache.seq_lens[b])
        O.latent_prefill(c.cache, b, X64, AK64, AV64)
        W.wsvd_prefill_append(L.ctx, L.desc, dev(codes), dev(s.view(np.uint16)), n_tok, b, AKd, AVd, L.cache)
        assert W.wsvd_check(L.ctx) == 0
        assert int(L.seq_lens[b]) == n0 + n_tok == int(c.cache.seq_lens[b])
    got, ref = run_attend(c, L)
    check_out(got, ref, sp.latent_dtype, f"attention after int8-x appends {name}")
    L.close()


def test_append_one_hot_token_and_capacity():
    """x = e_k appends row k of A (rounded to the storage format); a full sequence is left alone and flagged."""
    c = build_case("c2_small", batch=3)
    sp = c.sp
    L = layer_for(c)
    c.cache.seq_lens[:] = [5, c.t_cap, 0]
    L.upload(c.cache)
    x = np.zeros((3, sp.d_model), np.float32); x[0, 17] = 1; x[1, 3] = 1; x[2, 400] = 1
    st = L.append(as_dtype_dev(x, "bf16"), None, L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16"))
    assert st == 5, "capacity overflow must be reported by wsvd_check"
    assert L.seq_lens.cpu().numpy().tolist() == [6, c.t_cap, 1]
    assert W.wsvd_check(L.ctx) == 0, "error word must clear after being read"
    for b, e, t in ((0, 17, 5), (2, 400, 0)):
        gk, _, _ = L.download(0, t, 1); gv, _, _ = L.download(1, t, 1)
        assert (gk[b, :, 0] == O.bf16_bits_from_f32(c.AK[:, e])).all()
        assert (gv[b, :, 0] == O.bf16_bits_from_f32(c.AV[:, e])).all()
    gk, _, _ = L.download(0, 0, c.t_cap)
    assert (gk[1] == c.cache.k[1]).all(), "a sequence at capacity must not be modified"
    L.close()


def test_host_side_errors():
    c = build_case("c3_small")
    L = layer_for(c)
    d = L.desc
    bad = W.layer_desc(d.batch, 5, 4, 128, 512, 32, L.t_cap, "i8", "bf16", "bf16", "i8")
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_cache_bytes(bad)
    assert e.value.status == 2
    bad = W.layer_desc(d.batch, 4, 4, 128, 512, 32, L.t_cap + 1, "i8", "bf16", "bf16", "i8")
    with pytest.raises(W.WsvdError):
        W.wsvd_cache_bytes(bad)
    bad = W.layer_desc(d.batch, 4, 4, 128, 512, 32, L.t_cap, "i8", "f32", "bf16", "i8")
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_workspace_bytes(bad)
    assert e.value.status == 3
    q = torch.zeros((d.batch, 4, 128), dtype=torch.int8, device="cuda")
    with pytest.raises(W.WsvdError) as e:     # NULL q_scale with int8 queries
        W.wsvd_decode_attn(L.ctx, d, q, None, L.k_codes, L.k_codes, L.cache, 10, L.out)
    assert e.value.status == 1
    with pytest.raises(W.WsvdError) as e:     # max_seq_len beyond capacity
        W.wsvd_decode_attn(L.ctx, d, q, L.k_meta, L.k_codes, L.k_codes, L.cache, L.t_cap + 1, L.out)
    assert e.value.status == 5
    with pytest.raises(W.WsvdError) as e:     # misaligned pointer
        W.wsvd_decode_attn(L.ctx, d, q.data_ptr() + 1, L.k_meta, L.k_codes, L.k_codes, L.cache, 10, L.out)
    assert e.value.status == 4
    L.close()


# ------------------------------------------------------------------------------------------ bf16 output
BF16_OUT = [("c1", dict(batch=3, context=70)), ("c2_small", dict()), ("c3_small", dict()), ("c3_small", dict(n_q_heads=16, n_kv_heads=4)),
            ("c3_small", dict(context=2000, batch=2)), ("c4_small", dict()), ("c5_small", dict(context=2000)),
            ("c3_small", dict(rank=128, d_head=128))]


@pytest.mark.parametrize("name,over", BF16_OUT, ids=[f"{n}-{'-'.join(f'{k}{v}' for k, v in o.items())}" for n, o in BF16_OUT])
def test_attention_bf16_output_is_the_rounded_fp32_output(name, over):
    """out_dtype = BF16: every kernel rounds the value it would have stored as fp32 (round to nearest even), so the
    result must be the rounded fp32 result bit for bit; sequences of length 0 give zeros."""
    c = build_case(name, **over)
    sp = c.sp
    c.cache.seq_lens[0] = 0
    L = layer_for(c); L.upload(c.cache)
    got32, ref = run_attend(c, L)
    check_out(got32, ref, sp.latent_dtype, f"fp32 out {name}{over}")
    xdt = "f32" if sp.factor_dtype == "f32" else "bf16"
    desc16 = W.layer_desc(sp.batch, sp.n_q_heads, sp.n_kv_heads, sp.d_head, sp.d_model, sp.rank, L.desc.t_cap, sp.latent_dtype,
                          sp.factor_dtype, xdt, sp.q_dtype, "bf16", c.sm_scale)
    qd, qs, _ = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, sp.factor_dtype), as_dtype_dev(c.BV, sp.factor_dtype)
    out16 = torch.full((sp.batch, sp.n_q_heads, sp.d_head), float("nan"), dtype=torch.bfloat16, device="cuda")
    W.wsvd_decode_attn(L.ctx, desc16, qd, qs, BKd, BVd, L.cache, int(c.cache.seq_lens.max()), out16)
    assert W.wsvd_check(L.ctx) == 0
    want = torch.from_numpy(got32.astype(np.float32)).to(torch.bfloat16)
    assert (out16.cpu().view(torch.int16) == want.view(torch.int16)).all()
    assert (out16[0] == 0).all()
    if sp.latent_dtype == "i8" and sp.rank <= 64 and sp.n_q_heads // sp.n_kv_heads <= 4:
        # the rotary variant and the decode step (projection launch + attention launch that finishes the row)
        L.out.fill_(float("nan"))
        W.wsvd_decode_attn_rope(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, int(c.cache.seq_lens.max()), 10000.0, L.out)
        out16.fill_(float("nan"))
        W.wsvd_decode_attn_rope(L.ctx, desc16, qd, qs, BKd, BVd, L.cache, int(c.cache.seq_lens.max()), 10000.0, out16)
        assert W.wsvd_check(L.ctx) == 0
        assert (out16.cpu().view(torch.int16) == L.out.cpu().to(torch.bfloat16).view(torch.int16)).all()
        AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
        xd = as_dtype_dev(WI.bf16_exact(c.x_new[0]), "bf16")
        lens0 = L.seq_lens.clone()
        L.out.fill_(float("nan"))
        W.wsvd_decode_step(L.ctx, L.desc, xd, None, AKd, AVd, qd, qs, BKd, BVd, L.cache, int(c.cache.seq_lens.max()) + 1, L.out)
        L.seq_lens.copy_(lens0)
        out16.fill_(float("nan"))
        W.wsvd_decode_step(L.ctx, desc16, xd, None, AKd, AVd, qd, qs, BKd, BVd, L.cache, int(c.cache.seq_lens.max()) + 1, out16)
        assert W.wsvd_check(L.ctx) == 0
        assert (out16.cpu().view(torch.int16) == L.out.cpu().to(torch.bfloat16).view(torch.int16)).all()
    # the prompt kernels write fp32 only
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_prefill_attn(L.ctx, desc16, qd, 1, 0, BKd, BVd, L.cache, int(c.cache.seq_lens.max()), out16)
    assert e.value.status == W.E_UNSUPPORTED
    L.close()


# ------------------------------------------------------------------------------------------ rotary variant
ROPE_CASES = [
    ("c3_small", dict()),                                     # rank 32, head dim 128, int8 query
    ("c3_small", dict(q_dtype="f32", context=90)),
    ("c3_small", dict(context=2000, batch=2)),                # several chunks, long distances
    ("c3_small", dict(d_head=64)),                            # head dim 64
    ("c3_small", dict(n_q_heads=8, n_kv_heads=4)),            # two query heads per kv head
    ("c3_small", dict(n_q_heads=16, n_kv_heads=4, q_dtype="bf16", context=130)),   # four
    ("c3_small", dict(rank=64, context=700)),                 # rank 64
    ("c5_small", dict(n_q_heads=4, n_kv_heads=2, context=200)),    # rank 64, two query heads per kv head
    ("c5_small", dict(context=200)),                          # rank 64, G = 7: launches over head groups of 2, 2, 2, 1
    ("c3_small", dict(n_q_heads=28, n_kv_heads=4)),           # rank 32, G = 7: head groups of 4 and 3
    ("c3_small", dict(n_q_heads=20, n_kv_heads=4, context=2000, batch=2)),   # G = 5 (4 + 1) over several chunks
    ("c3_small", dict(n_q_heads=32, n_kv_heads=4, d_head=64, context=500)),  # G = 8 (4 + 4), head dim 64
    ("c4_small", dict()),                                     # int4 latents (ragged lengths): codes minus zero point as operands
    ("c4_small", dict(n_q_heads=8, n_kv_heads=4, q_dtype="bf16")),
    ("c4_small", dict(n_q_heads=28, n_kv_heads=4, d_head=64, context=1500, ragged=())),   # int4, G = 7, head dim 64, several chunks
]


@pytest.mark.parametrize("name,over", ROPE_CASES, ids=[f"{n}-{'-'.join(f'{k}{v}' for k, v in o.items())}" for n, o in ROPE_CASES])
def test_attention_rope_small(name, over):
    """Reconstruct-rotate-attend against the oracle that forms K = C B_K, rotates keys and query, and attends."""
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    got = L.attend_rope(qd, qs, BKd, BVd, int(c.cache.seq_lens.max()), 10000.0)
    ref = O.decode_attn_rope_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale, 10000.0)
    check_out(got, ref, "rope", f"rope {name}{over}")
    plain = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    assert np.abs(ref - plain).max() > 1e-2, "the case does not exercise the rotation"
    L.close()


def test_attention_rope_edge_lengths_and_other_base():
    lens = [0, 1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 640]
    c = build_case("c3_small", batch=len(lens), context=640, ragged=(), extra_cap=0, steps=1)
    for b, n in enumerate(lens):
        c.cache.seq_lens[b] = n
    L = layer_for(c); L.upload(c.cache)
    qd, qs, q64 = q_to_device(c.q32[0], c.sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    for base in (10000.0, 500000.0):
        got = L.attend_rope(qd, qs, BKd, BVd, 640, base)
        ref = O.decode_attn_rope_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale, base)
        assert (got[0] == 0).all()
        check_out(got, ref, "rope", f"rope edges base={base}")
    # unsupported combinations are refused, not mis-computed
    c4 = build_case("c2_small")
    L4 = layer_for(c4); L4.upload(c4.cache)
    qd4, qs4, _ = q_to_device(c4.q32[0], c4.sp.q_dtype)
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_decode_attn_rope(L4.ctx, L4.desc, qd4, qs4, BKd, BVd, L4.cache, 64, 10000.0, L4.out)
    assert e.value.status == W.E_UNSUPPORTED
    L4.close(); L.close()


# ------------------------------------------------------------------------------------------ fused decode step
STEP_CASES = [
    ("c3_small", dict(), 2),                                      # int8, one chunk per sequence
    ("c3_small", dict(context=2000, batch=2), 2),                 # several chunks: split merge + late tile
    ("c3_small", dict(rank=64, context=700), 2),                  # rank 64
    ("c3_small", dict(n_q_heads=8, n_kv_heads=4, q_dtype="f32"), 2),   # two query heads per kv head
    ("c4_small", dict(), 2),                                      # int4, ragged lengths
    ("c2_small", dict(), 1),                                      # bf16 latents: no single-launch kernel, two launches
    ("c1", dict(batch=3, context=70), 1),                         # fp32: likewise
    ("c3_small", dict(), 0),                                      # the append launch and the attention launch
    # mode 3: projection launch + attention launch that sums the slices, quantises, stores and patches the row
    ("c3_small", dict(), 3),
    ("c3_small", dict(context=2000, batch=2), 3),                 # several chunks: the row's chunk finishes it
    ("c3_small", dict(rank=64, context=700), 3),
    ("c3_small", dict(n_q_heads=8, n_kv_heads=4, q_dtype="f32"), 3),
    ("c5_small", dict(n_q_heads=8, n_kv_heads=2), 3),             # rank 64, four query heads per kv head
    ("c3_small", dict(batch=21, context=130), 3),                 # two groups of sequences in the projection launch
    ("c3_small", dict(), -1),                                     # whatever the library does by default
    ("c4_small", dict(), -1),
    # -2: the defaults, the library's own chunk policy included (2000 rows of a few sequences stay one chunk)
    ("c3_small", dict(context=2000, batch=2), -2),
    ("c4_small", dict(context=2000, batch=2), -2),
    ("c5_small", dict(context=2000, batch=2), -2),
]


def _set_step_mode(ctx, mode):
    """0 two launches, 1 / 2 the single-launch kernel (where it exists / or refuse), 3 the deferred-row pair of launches."""
    if mode < 0:
        return                                          # the context's defaults
    W.wsvd_ctx_set_option(ctx, "fused_step", mode if mode in (1, 2) else 0)
    W.wsvd_ctx_set_option(ctx, "step_deferred", 2 if mode == 3 else 0)


@pytest.mark.parametrize("name,over,mode", STEP_CASES, ids=[f"{n}-{'-'.join(f'{k}{v}' for k, v in o.items())}" for n, o, _ in STEP_CASES])
def test_decode_step_matches_oracle(name, over, mode):
    """wsvd_decode_step = append + attention (including the appended row).  mode 2 insists on the single-launch
    kernel, mode 1 takes it where it exists, mode 0 is the default pair of launches.
    Three consecutive steps on the GPU's own cache; each compared with the oracle doing the same on its cache."""
    c = build_case(name, steps=3, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    xdt = "f32" if sp.factor_dtype == "f32" else "bf16"
    AKd, AVd = L.pack_A(c.AK, sp.factor_dtype), L.pack_A(c.AV, sp.factor_dtype)
    BKd, BVd = as_dtype_dev(c.BK, sp.factor_dtype), as_dtype_dev(c.BV, sp.factor_dtype)
    AK64, AV64, BK64, BV64 = (a.astype(np.float64) for a in (c.AK, c.AV, c.BK, c.BV))
    flips = 0
    try:
        _set_step_mode(L.ctx, mode)
        if mode == -2:
            W.wsvd_ctx_set_option(L.ctx, "min_chunk", 0)
        for step in range(3):
            x = c.x_new[step]
            if xdt == "bf16":
                x = WI.bf16_exact(x)
            before = c.cache.seq_lens.copy()
            x64 = x.astype(np.float64)
            cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
            O.latent_append(c.cache, x64, AK64, AV64)
            qd, qs, q64 = q_to_device(c.q32[step], sp.q_dtype)
            ref = O.decode_attn_reconstructed(c.cache, q64, BK64, BV64, c.sm_scale)
            got, st = L.step(as_dtype_dev(x, xdt), AKd, AVd, qd, qs, BKd, BVd, int(c.cache.seq_lens.max()))
            assert st == 0, W.status_str(st)
            assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all(), "seq_lens not advanced by exactly one"
            flips += _append_compare(L, c.cache, cK, cV, before, sp.latent_dtype)
            check_out(got, ref, sp.latent_dtype, f"step {step} {name}{over}")
            if mode == 3:
                # the step's second launch once more (measurement aid): same rows stored again, same output, bit for bit
                planes = [t.clone() for t in (L.k_codes, L.v_codes, L.k_meta, L.v_meta)]
                out2 = torch.full_like(L.out, float("nan"))
                W.wsvd_test_step_attention(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, int(c.cache.seq_lens.max()), out2)
                assert W.wsvd_check(L.ctx) == 0
                assert (out2.cpu().numpy().astype(np.float64) == got).all()
                assert all((a == b).all() for a, b in zip(planes, (L.k_codes, L.v_codes, L.k_meta, L.v_meta)))
                assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
            L.upload(c.cache)      # continue from the oracle's cache so that later steps compare like with like
    finally:
        _set_step_mode(L.ctx, -1 if mode < 0 else 0)
        W.wsvd_ctx_set_option(L.ctx, "min_chunk", 256)
    assert flips <= max(2, 2 * sp.batch * sp.n_kv_heads * sp.rank * 3 // 500)
    L.close()


def test_decode_step_tile_boundaries_and_capacity():
    """The appended row starts a new 64-row tile, ends one, starts a new chunk, is the first row ever; one sequence is
    full (left alone and flagged, attended as it is).  Fused kernel; the unfused pair of calls must agree closely."""
    lens = [0, 1, 62, 63, 64, 65, 127, 128, 255, 256, 257, 511, 512, 639, 640]
    c = build_case("c3_small", batch=len(lens), context=640, ragged=(), extra_cap=0, steps=1)
    for b, n in enumerate(lens):
        c.cache.seq_lens[b] = n
    sp = c.sp
    assert c.t_cap == 640 + 64
    c.cache.seq_lens[-1] = c.t_cap                      # full
    L = layer_for(c); L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    x = WI.bf16_exact(c.x_new[0]); x64 = x.astype(np.float64)
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    outs = []
    for mode in (2, 3, 0):
        L.upload(c.cache)
        _set_step_mode(L.ctx, mode)
        try:
            got, st = L.step(as_dtype_dev(x, "bf16"), AKd, AVd, qd, qs, BKd, BVd, c.t_cap)
        finally:
            _set_step_mode(L.ctx, 0)
        assert st == W.E_CAPACITY
        lens_after = L.seq_lens.cpu().numpy()
        assert (lens_after[:-1] == np.array(lens[:-1]) + 1).all() and lens_after[-1] == c.t_cap
        outs.append(got)
    oc = c.cache
    full_rows = (oc.k[-1].copy(), oc.v[-1].copy())
    ov = O.latent_append(oc, x64, c.AK.astype(np.float64), c.AV.astype(np.float64))
    assert ov[-1] and not ov[:-1].any()
    assert (oc.k[-1] == full_rows[0]).all() and (oc.v[-1] == full_rows[1]).all()
    ref = O.decode_attn_reconstructed(oc, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    for got in outs:
        check_out(got, ref, "i8", "step at tile boundaries")
    for o in outs[:-1]:
        assert np.abs(o - outs[-1]).max() <= 1e-5 * np.abs(outs[-1]).max()
    L.close()


# ------------------------------------------------------------------------------------------ the five workloads, full size
def test_config1_fp32_full():
    c = build_case("c1")
    L = layer_for(c, min_chunk=0); L.upload(c.cache)
    got, ref = run_attend(c, L)                       # 256 rows, no append
    check_out(got, ref, "f32", "c1 attend(256)")
    x = c.x_new[0]
    O.latent_append(c.cache, x.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
    assert L.append(dev(x), None, L.pack_A(c.AK, "f32"), L.pack_A(c.AV, "f32")) == 0
    qd, qs, q64 = q_to_device(c.q32[0], "f32")
    got = L.attend(qd, qs, dev(c.BK), dev(c.BV), 257)  # GPU-appended row 256 included
    ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    check_out(got, ref, "f32", "c1 append+attend(257)")
    L.close()


def test_config2_bf16_32_steps():
    """32 consecutive (append, attend) steps on the GPU's own cache; every step compared with the oracle
    running the same steps on its cache."""
    c = build_case("c2")
    sp = c.sp
    L = layer_for(c, min_chunk=0); L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    AK64, AV64, BK64, BV64 = (a.astype(np.float64) for a in (c.AK, c.AV, c.BK, c.BV))
    worst = 0.0
    for step in range(sp.steps):
        x = WI.bf16_exact(c.x_new[step])
        O.latent_append(c.cache, x.astype(np.float64), AK64, AV64)
        assert L.append(as_dtype_dev(x, "bf16"), None, AKd, AVd) == 0
        qd, qs, q64 = q_to_device(c.q32[step], "bf16")
        got = L.attend(qd, qs, BKd, BVd, 640 + step + 1)
        ref = O.decode_attn_reconstructed(c.cache, q64, BK64, BV64, c.sm_scale)
        a, r, l2 = err_stats(got, ref)
        worst = max(worst, l2)
        assert a <= 2e-2 and l2 <= 1e-3, f"step {step}: max_abs {a} rel_l2 {l2}"
    assert L.seq_lens.cpu().numpy().tolist() == [672]
    print(f"c2: worst rel L2 over 32 steps = {worst:.3e}", flush=True)
    L.close()


def test_config3_int8_full():
    c = build_case("c3")
    L = layer_for(c, min_chunk=0); L.upload(c.cache)
    got, ref = run_attend(c, L)
    check_out(got, ref, "i8", "c3 full")
    L.close()


def test_config3_int8_append_and_step_full():
    """The cache update of the batched int8 workload at its full shape (16 sequences, d_model 4096, 32 kv heads: the
    launch the benchmark times, several d_model slices merged through the workspace), rows compared with the oracle's;
    then a whole wsvd_decode_step at the same shape, all 512 heads against the materialising oracle."""
    c = build_case("c3", steps=2)
    sp = c.sp
    L = layer_for(c, min_chunk=0); L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    AK64, AV64, BK64, BV64 = (a.astype(np.float64) for a in (c.AK, c.AV, c.BK, c.BV))
    # 1. append alone
    x = WI.bf16_exact(c.x_new[0]); x64 = x.astype(np.float64)
    before = c.cache.seq_lens.copy()
    cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
    assert not O.latent_append(c.cache, x64, AK64, AV64).any()
    assert L.append(as_dtype_dev(x, "bf16"), None, AKd, AVd) == 0
    assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    flips = _append_compare(L, c.cache, cK, cV, before, "i8")
    print(f"c3 full append: boundary flips accepted = {flips} of {2 * sp.batch * sp.n_kv_heads * sp.rank} codes", flush=True)
    assert flips <= 8
    # the rows before the new one are untouched
    for plane, codes in ((0, c.cache.k), (1, c.cache.v)):
        gc, _, _ = L.download(plane, 0, int(before.min()))
        assert (gc.reshape(codes[:, :, :int(before.min())].shape) == codes[:, :, :int(before.min())]).all()
    # 2. a whole decode step on top (from the oracle's cache, so that both sides attend over the same rows)
    L.upload(c.cache)
    x = WI.bf16_exact(c.x_new[1]); x64 = x.astype(np.float64)
    before = c.cache.seq_lens.copy()
    cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
    assert not O.latent_append(c.cache, x64, AK64, AV64).any()
    qd, qs, q64 = q_to_device(c.q32[1], sp.q_dtype)
    got, st = L.step(as_dtype_dev(x, "bf16"), AKd, AVd, qd, qs, BKd, BVd, int(c.cache.seq_lens.max()))
    assert st == 0, W.status_str(st)
    assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    flips = _append_compare(L, c.cache, cK, cV, before, "i8")
    assert flips <= 8
    ref = O.decode_attn_reconstructed(c.cache, q64, BK64, BV64, c.sm_scale)
    check_out(got, ref, "i8", "c3 full decode step (append + attention)")
    L.close()


def test_config3_int8_full_rope():
    """The rotary variant at the full batched shape, in the launch configuration the benchmark times; the oracle forms
    and rotates the keys of a sample of (sequence, head) pairs."""
    c = build_case("c3")
    sp = c.sp
    L = layer_for(c, min_chunk=0); L.upload(c.cache)
    rng = np.random.default_rng(33)
    heads = [(int(b), int(h)) for b, h in zip(rng.integers(0, sp.batch, 96), rng.integers(0, sp.n_q_heads, 96))]
    heads += [(0, 0), (sp.batch - 1, sp.n_q_heads - 1)]
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    got = L.attend_rope(qd, qs, BKd, BVd, int(c.cache.seq_lens.max()), 10000.0)
    ref = O.decode_attn_rope_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale,
                                           10000.0, heads=heads)
    check_out(got, ref, "rope", "c3 full, rotary, sampled heads")
    assert np.isfinite(got).all()
    L.close()


def test_config4_int4_append_and_step_full():
    """The cache update of the ragged int4 workload at its full shape (64 sequences, d_model 4096, 32 kv heads: the launch
    the benchmark times - two groups of 32 sequences, a finisher and one helper per (plane, kv head) and group), rows
    compared with the oracle's; then a whole wsvd_decode_step on top, sampled heads against the materialising oracle."""
    c = build_case("c4", steps=2)
    sp = c.sp
    L = layer_for(c, min_chunk=0); L.upload(c.cache)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    AK64, AV64, BK64, BV64 = (a.astype(np.float64) for a in (c.AK, c.AV, c.BK, c.BV))
    x = WI.bf16_exact(c.x_new[0]); x64 = x.astype(np.float64)
    before = c.cache.seq_lens.copy()
    cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
    assert not O.latent_append(c.cache, x64, AK64, AV64).any()
    assert L.append(as_dtype_dev(x, "bf16"), None, AKd, AVd) == 0
    assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    flips = _append_compare(L, c.cache, cK, cV, before, "i4")
    print(f"c4 full append: boundary flips accepted = {flips} of {2 * sp.batch * sp.n_kv_heads * sp.rank} codes", flush=True)
    assert flips <= 16
    L.upload(c.cache)
    x = WI.bf16_exact(c.x_new[1]); x64 = x.astype(np.float64)
    before = c.cache.seq_lens.copy()
    cK = O.project_latents(x64, AK64); cV = O.project_latents(x64, AV64)
    assert not O.latent_append(c.cache, x64, AK64, AV64).any()
    qd, qs, q64 = q_to_device(c.q32[1], sp.q_dtype)
    got, st = L.step(as_dtype_dev(x, "bf16"), AKd, AVd, qd, qs, BKd, BVd, int(c.cache.seq_lens.max()))
    assert st == 0, W.status_str(st)
    assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    flips = _append_compare(L, c.cache, cK, cV, before, "i4")
    assert flips <= 16
    rng = np.random.default_rng(14)
    heads = sorted(set((int(b), int(h)) for b, h in zip(rng.integers(0, sp.batch, 48), rng.integers(0, sp.n_q_heads, 48))))
    ref = O.decode_attn_reconstructed(c.cache, q64, BK64, BV64, c.sm_scale, heads=heads)
    m = ~np.isnan(ref)
    a, _, l2 = err_stats(got[m], ref[m])
    print(f"c4 full decode step, {len(heads)} sampled (sequence, head) pairs: max_abs={a:.3e} rel_l2={l2:.3e}", flush=True)
    assert np.isfinite(got).all() and a <= 2e-2 and l2 <= 1e-3
    L.close()


def test_config4_int4_ragged_full():
    c = build_case("c4")
    sp = c.sp
    L = layer_for(c, min_chunk=0); L.upload(c.cache)
    rng = np.random.default_rng(4)
    heads = [(int(b), int(h)) for b, h in zip(rng.integers(0, sp.batch, 192), rng.integers(0, sp.n_q_heads, 192))]
    heads += [(int(np.argmin(c.lens)), 0), (int(np.argmax(c.lens)), sp.n_q_heads - 1)]
    got, ref = run_attend(c, L, heads=heads)
    check_out(got, ref, "i4", "c4 sampled (reconstructed oracle)")
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    ref_all = O.decode_attn_absorbed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    m = ~np.isnan(ref)
    assert np.abs(ref_all[m] - ref[m]).max() <= 1e-9 * np.abs(ref[m]).max()
    check_out(got, ref_all, "i4", "c4 all heads (absorbed oracle, agreed with the reconstructed one on the sample)")
    L.close()
