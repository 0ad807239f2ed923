"""GPU parity tests for the rest of the decoding pipeline (Section 3.4): the two offline folds, the attention that
takes the Q latent and returns the latent-space output, the row kernels of the quantised decoder layer, and the
layer as a whole against the oracle's ``decoder_layer_w4a8``."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
import wsvd_inputs as WI
from cases import build_case
from harness import as_dtype_dev, check_i8_rows, dev, err_stats
from test_gpu_parity import _append_compare, check_out, layer_for

pytestmark = pytest.mark.gpu

u16 = lambda a: dev(np.asarray(a, np.float16).view(np.uint16))


def _codes_close(got_codes, got_scale, ref_codes, ref_scale, values, what, max_flip_frac=2e-3):
    """int8 rows produced from fp32 values that differ from the oracle's in the last bits (a different summation order,
    the hardware's reciprocal square root and logistic): every row is compared; a scale may differ only between fp16
    neighbours with the row maximum on their rounding boundary, a code only by one step next to a .5 boundary
    (harness.check_i8_rows).  ref_codes / ref_scale are the oracle's and must be what its quantiser gives for values."""
    rc, rs = O.quantize_act_i8(np.asarray(values, np.float32))
    assert (rc == np.asarray(ref_codes)).all() and (rs.view(np.uint16) == np.asarray(ref_scale, np.float16).view(np.uint16)).all()
    flips = check_i8_rows(got_codes, got_scale, np.asarray(values, np.float32).astype(np.float64), what, code_tol=2e-3, scale_tol=2e-5)
    assert flips <= max(2, int(max_flip_frac * np.asarray(got_codes).size)), f"{what}: {flips} accepted differences are too many to be boundary cases"
    return flips


# ------------------------------------------------------------------------------------------ folds
@pytest.mark.parametrize("name,rq,over", [("c3_small", 32, dict()), ("c3_small", 24, dict(n_q_heads=8, n_kv_heads=4)),
                                          ("c5_small", 64, dict()), ("c1", 16, dict())])
def test_folds_match_oracle(name, rq, over):
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c)
    _, BQ = WI.lowrank_q_factors(sp, rq)
    fd = sp.factor_dtype
    rng = np.random.default_rng(3)
    WO = (rng.standard_normal((sp.d_model, sp.n_q_heads * sp.d_head)) / np.sqrt(sp.n_q_heads * sp.d_head)).astype(np.float32)
    M = torch.empty((sp.n_q_heads, rq, sp.rank), dtype=torch.float32, device="cuda")
    WOf = torch.empty((sp.d_model, sp.n_q_heads * sp.rank), dtype=torch.float32, device="cuda")
    W.wsvd_fold_qk(L.ctx, L.desc, as_dtype_dev(BQ, fd), rq, as_dtype_dev(c.BK, fd), M)
    W.wsvd_fold_vo(L.ctx, L.desc, as_dtype_dev(c.BV, fd), dev(WO), WOf)
    torch.cuda.synchronize()
    refM = O.fold_qk(BQ.astype(np.float64), c.BK.astype(np.float64))
    refW = O.fold_vo(c.BV.astype(np.float64), WO.astype(np.float64), sp.n_q_heads)
    for what, got, ref in (("B_Q B_K^T", M.cpu().numpy(), refM), ("W_O with B_V folded in", WOf.cpu().numpy(), refW)):
        a, rmax, l2 = err_stats(got.astype(np.float64), ref)
        print(f"fold {what}: max_abs={a:.3e} rel_l2={l2:.3e}", flush=True)
        assert l2 <= 1e-6 and a <= 1e-5 * np.abs(ref).max()
    L.close()


# ------------------------------------------------------------------------------------------ attention, latent in / out
def _latent_q(c, rq, step=0):
    sp = c.sp
    AQ, BQ = WI.lowrank_q_factors(sp, rq)
    cQ = np.einsum("be,hej->bhj", c.x_new[step].astype(np.float64), AQ.astype(np.float64)).astype(np.float32)
    return cQ, BQ


LATENT_CASES = [
    ("c3_small", 32, dict()),                                               # rank 32, one query head per kv head
    ("c3_small", 20, dict(context=2000, batch=2)),                          # rq < r, several chunks
    ("c3_small", 32, dict(n_q_heads=8, n_kv_heads=4)),
    ("c3_small", 48, dict(n_q_heads=16, n_kv_heads=4, context=130)),        # four heads per kv head, rq > r
    ("c3_small", 64, dict(rank=64, context=700)),
    ("c5_small", 64, dict(n_q_heads=8, n_kv_heads=2, context=200)),         # rank 64, four heads per kv head
    ("c4_small", 32, dict()),                                               # int4 latents, ragged
    ("c4_small", 7, dict(n_q_heads=12, n_kv_heads=4)),                      # int4, three heads per kv head, odd rq
    ("c5_small", 64, dict()),                                               # rank 64, seven heads per kv head
    ("c3_small", 32, dict(n_q_heads=20, n_kv_heads=4, context=900)),        # rank 32, five heads per kv head
    ("c3_small", 48, dict(n_q_heads=16, n_kv_heads=2, context=70)),         # eight heads per kv head
    ("c5_small", 13, dict(n_q_heads=12, n_kv_heads=2, context=2500, batch=2)),   # six, several chunks
    ("c4_small", 32, dict(n_q_heads=28, n_kv_heads=4)),                     # int4, seven heads per kv head: 4 + 3 in two launches
    ("c4_small", 20, dict(n_q_heads=10, n_kv_heads=2, context=2000, batch=2, ragged=())),   # int4, five, several chunks
]


@pytest.mark.parametrize("name,rq,over", LATENT_CASES, ids=[f"{n}-rq{q}-{'-'.join(f'{k}{v}' for k, v in o.items())}" for n, q, o in LATENT_CASES])
def test_attention_latent_small(name, rq, over):
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    cQ, BQ = _latent_q(c, rq)
    BK64, BV64 = c.BK.astype(np.float64), c.BV.astype(np.float64)
    M64 = O.fold_qk(BQ.astype(np.float64), BK64)
    u = torch.empty((sp.batch, sp.n_q_heads, sp.rank), dtype=torch.float32, device="cuda")
    W.wsvd_decode_attn_latent(L.ctx, L.desc, dev(cQ), rq, dev(M64.astype(np.float32)), L.cache, int(c.cache.seq_lens.max()), u)
    assert W.wsvd_check(L.ctx) == 0
    got = u.cpu().numpy().astype(np.float64)
    ref_u = O.decode_attn_latent_out(c.cache, cQ.astype(np.float64), M64.astype(np.float32).astype(np.float64), c.sm_scale)
    check_out(got, ref_u, sp.latent_dtype, f"latent attention {name} rq={rq} {over}")
    # against the pipeline in the paper's order: up-project the Q latent, attend over reconstructed K and V
    o_ref = O.decode_attn_lowrank_q(c.cache, cQ.astype(np.float64), BQ.astype(np.float64), BK64, BV64, c.sm_scale)
    G = sp.n_q_heads // sp.n_kv_heads
    o_got = np.einsum("bhj,hjc->bhc", got, BV64[np.arange(sp.n_q_heads) // G])
    check_out(o_got, o_ref, sp.latent_dtype, "  ... times B_V, against the unfolded pipeline")
    L.close()


def test_attention_latent_edge_lengths_and_errors():
    lens = [0, 1, 2, 63, 64, 65, 127, 128, 129, 511, 512, 640]
    c = build_case("c3_small", batch=len(lens), context=640, ragged=(), extra_cap=0, steps=1)
    for b, n in enumerate(lens):
        c.cache.seq_lens[b] = n
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    cQ, BQ = _latent_q(c, 32)
    M32 = O.fold_qk(BQ.astype(np.float64), c.BK.astype(np.float64)).astype(np.float32)
    u = torch.full((sp.batch, sp.n_q_heads, sp.rank), 7.0, dtype=torch.float32, device="cuda")
    W.wsvd_decode_attn_latent(L.ctx, L.desc, dev(cQ), 32, dev(M32), L.cache, 640, u)
    got = u.cpu().numpy().astype(np.float64)
    ref = O.decode_attn_latent_out(c.cache, cQ.astype(np.float64), M32.astype(np.float64), c.sm_scale)
    assert (got[0] == 0).all()
    check_out(got, ref, "i8", "latent attention, edge lengths")
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_decode_attn_latent(L.ctx, L.desc, dev(cQ), 65, dev(M32), L.cache, 640, u)
    assert e.value.status == W.E_SHAPE
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_decode_attn_latent(L.ctx, L.desc, dev(cQ), 32, None, L.cache, 640, u)
    assert e.value.status == W.E_NULL
    L.close()
    c2 = build_case("c2_small")                        # bf16 latents: no such kernel
    L2 = layer_for(c2); L2.upload(c2.cache)
    u2 = torch.empty((c2.sp.batch, c2.sp.n_q_heads, c2.sp.rank), dtype=torch.float32, device="cuda")
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_decode_attn_latent(L2.ctx, L2.desc, dev(cQ), 32, dev(M32), L2.cache, 64, u2)
    assert e.value.status == W.E_UNSUPPORTED
    L2.close()


# ------------------------------------------------------------------------------------------ row kernels
@pytest.mark.parametrize("rows,cols,add", [(3, 512, False), (16, 4096, True), (5, 11008, True), (2, 16384, False), (1, 4, True)])
def test_rmsnorm_quant_matches_oracle(rows, cols, add):
    rng = np.random.default_rng(rows * 131 + cols)
    x = (rng.standard_normal((rows, cols)) * np.exp(rng.standard_normal((rows, 1)))).astype(np.float32)
    y = (rng.standard_normal((rows, cols)) * 0.3).astype(np.float32) if add else None
    g = (1 + 0.1 * rng.standard_normal(cols)).astype(np.float32)
    eps = 1e-5
    ctx = W.wsvd_create(0)
    xo = torch.empty((rows, cols), dtype=torch.float32, device="cuda") if add else None
    codes = torch.empty((rows, cols), dtype=torch.int8, device="cuda"); sc = torch.empty(rows, dtype=torch.int16, device="cuda")
    W.wsvd_rmsnorm_quant_i8(ctx, dev(x), dev(y) if add else None, dev(g), eps, rows, cols, xo, codes, sc)
    torch.cuda.synchronize()
    r = (x.astype(np.float64) + y.astype(np.float64)).astype(np.float32) if add else x
    if add:
        assert (xo.cpu().numpy() == r).all(), "residual sum must be the correctly rounded fp32 sum"
    h = O.rmsnorm(r.astype(np.float64), g.astype(np.float64), eps)
    rc, rs = O.quantize_act_i8(h.astype(np.float32))
    flips = _codes_close(codes.cpu().numpy(), sc.cpu().numpy(), rc, rs, h, f"rmsnorm {rows}x{cols}")
    print(f"rmsnorm {rows}x{cols} add={add}: boundary flips accepted = {flips}", flush=True)
    # the de-quantised result is the normalised row within half a step
    deq = codes.cpu().numpy().astype(np.float64) * sc.cpu().numpy().view(np.float16).astype(np.float64)[:, None]
    assert (np.abs(deq - h) <= 0.51 * sc.cpu().numpy().view(np.float16).astype(np.float64)[:, None] + 1e-6).all()
    W.wsvd_destroy(ctx)


@pytest.mark.parametrize("rows,F", [(3, 1408), (16, 11008), (1, 4), (2, 16384)])
def test_swiglu_quant_matches_oracle(rows, F):
    rng = np.random.default_rng(rows * 17 + F)
    gu = (rng.standard_normal((rows, 2 * F)) * 2).astype(np.float32)
    gu[0, :4] = [0.0, -30.0, 30.0, -100.0]                 # saturating arguments of the logistic
    ctx = W.wsvd_create(0)
    codes = torch.empty((rows, F), dtype=torch.int8, device="cuda"); sc = torch.empty(rows, dtype=torch.int16, device="cuda")
    W.wsvd_swiglu_quant_i8(ctx, dev(gu), rows, F, codes, sc)
    torch.cuda.synchronize()
    a = O.silu(gu[:, :F].astype(np.float64)) * gu[:, F:].astype(np.float64)
    rc, rs = O.quantize_act_i8(a.astype(np.float32))
    flips = _codes_close(codes.cpu().numpy(), sc.cpu().numpy(), rc, rs, a, f"swiglu {rows}x{F}")
    print(f"swiglu {rows}x{F}: boundary flips accepted = {flips}", flush=True)
    W.wsvd_destroy(ctx)


def test_row_kernel_host_errors():
    ctx = W.wsvd_create(0)
    x = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
    c = torch.zeros((2, 64), dtype=torch.int8, device="cuda"); s = torch.zeros(2, dtype=torch.int16, device="cuda")
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_rmsnorm_quant_i8(ctx, x, x, x, 1e-5, 2, 64, None, c, s)          # residual given, no place for the sum
    assert e.value.status == W.E_NULL
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_rmsnorm_quant_i8(ctx, x, None, x, 1e-5, 2, 62, None, c, s)
    assert e.value.status == W.E_SHAPE
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_swiglu_quant_i8(ctx, x, 2, 16388, c, s)
    assert e.value.status == W.E_SHAPE
    W.wsvd_destroy(ctx)


# ------------------------------------------------------------------------------------------ the layer
class LayerWeights:
    pass


def build_layer_case(name, rq, d_ffn, layer=0, **over):
    """build_case plus everything a decoder layer needs: int4 stacked [A_Q; A_K; A_V], B_Q, the fold M (oracle side),
    int4 W'_O [E, Hq r], int4 [W_g; W_u] and W_d, two norm gains, and the fp32 residual-stream input."""
    c = build_case(name, layer=layer, **over)
    sp = c.sp
    w = LayerWeights()
    w.rq, w.F = rq, d_ffn
    n_qkv = sp.n_q_heads * rq + 2 * sp.n_kv_heads * sp.rank
    w.qkv = WI.int4_weight(sp, n_qkv, 4, layer)
    _, w.BQ = WI.lowrank_q_factors(sp, rq, layer)
    w.M64 = O.fold_qk(w.BQ.astype(np.float64), c.BK.astype(np.float64))
    w.wo = WI.int4_weight(dataclasses.replace(sp, d_model=sp.n_q_heads * sp.rank), sp.d_model, 5, layer)
    w.gu = WI.int4_weight(sp, 2 * d_ffn, 6, layer)
    w.wd = WI.int4_weight(dataclasses.replace(sp, d_model=d_ffn), sp.d_model, 7, layer)
    w.g1, w.g2 = WI.norm_gains(sp, 0, layer), WI.norm_gains(sp, 1, layer)
    c.w = w
    c.x32 = c.x_new[0].astype(np.float32)
    return c


def oracle_layer(c):
    sp, w = c.sp, c.w
    return O.decoder_layer_w4a8(c.cache, c.x32, w.g1, w.g2, O.pack_w4(w.qkv[0]), w.qkv[1], w.M64.astype(np.float32).astype(np.float64),
                                O.pack_w4(w.wo[0]), w.wo[1], O.pack_w4(w.gu[0]), w.gu[1], O.pack_w4(w.wd[0]), w.wd[1],
                                sp.n_q_heads, w.rq, c.sm_scale, 1e-5)


class GpuLayer:
    """The GPU chain of one decoder layer: 10 launches through the C ABI, buffers allocated once."""

    def __init__(self, c, L, fold_on_gpu=True):
        sp, w = c.sp, c.w
        self.c, self.L = c, L
        B, E, Hq, Hkv, r, rq, F = sp.batch, sp.d_model, sp.n_q_heads, sp.n_kv_heads, sp.rank, w.rq, w.F
        self.dims = (B, E, Hq, Hkv, r, rq, F)
        f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
        i8 = lambda *s: torch.empty(s, dtype=torch.int8, device="cuda")
        i16 = lambda *s: torch.empty(s, dtype=torch.int16, device="cuda")
        self.wqkv, self.wqkv_s = dev(O.pack_w4(w.qkv[0])), u16(w.qkv[1])
        self.wo, self.wo_s = dev(O.pack_w4(w.wo[0])), u16(w.wo[1])
        self.wgu, self.wgu_s = dev(O.pack_w4(w.gu[0])), u16(w.gu[1])
        self.wd, self.wd_s = dev(O.pack_w4(w.wd[0])), u16(w.wd[1])
        self.g1, self.g2 = dev(w.g1), dev(w.g2)
        self.M = f32(Hq, rq, r)
        if fold_on_gpu:
            W.wsvd_fold_qk(L.ctx, L.desc, as_dtype_dev(w.BQ, sp.factor_dtype), rq, as_dtype_dev(c.BK, sp.factor_dtype), self.M)
        else:
            self.M.copy_(dev(w.M64.astype(np.float32)))
        self.h_codes, self.h_scale = i8(B, E), i16(B)
        self.cq, self.lat = f32(B, Hq * rq), f32(B, 2 * Hkv * r)
        self.u = f32(B, Hq, r)
        self.u_codes, self.u_scale = i8(B, Hq * r), i16(B)
        self.y, self.x1 = f32(B, E), f32(B, E)
        self.gu = f32(B, 2 * F)
        self.a_codes, self.a_scale = i8(B, F), i16(B)
        self.down, self.x2 = f32(B, E), f32(B, E)
        self.tail_codes, self.tail_scale = i8(B, E), i16(B)

    def run(self, x, max_seq_len):
        L = self.L
        B, E, Hq, Hkv, r, rq, F = self.dims
        ctx = L.ctx
        W.wsvd_rmsnorm_quant_i8(ctx, x, None, self.g1, 1e-5, B, E, None, self.h_codes, self.h_scale)
        W.wsvd_linear_w4a8_split(ctx, self.h_codes, self.h_scale, self.wqkv, self.wqkv_s, B, E, Hq * rq + 2 * Hkv * r, Hq * rq,
                                 self.cq, self.lat)
        W.wsvd_latent_store(ctx, L.desc, self.lat, self.lat[:, Hkv * r:], 2 * Hkv * r, L.cache)
        W.wsvd_decode_attn_latent(ctx, L.desc, self.cq, rq, self.M, L.cache, max_seq_len, self.u)
        W.wsvd_quantize_act_i8(ctx, self.u, W.F32, B, Hq * r, self.u_codes, self.u_scale)
        W.wsvd_linear_w4a8(ctx, self.u_codes, self.u_scale, self.wo, self.wo_s, B, Hq * r, E, self.y)
        W.wsvd_rmsnorm_quant_i8(ctx, x, self.y, self.g2, 1e-5, B, E, self.x1, self.h_codes, self.h_scale)
        W.wsvd_linear_w4a8(ctx, self.h_codes, self.h_scale, self.wgu, self.wgu_s, B, E, 2 * F, self.gu)
        W.wsvd_swiglu_quant_i8(ctx, self.gu, B, F, self.a_codes, self.a_scale)
        W.wsvd_linear_w4a8(ctx, self.a_codes, self.a_scale, self.wd, self.wd_s, B, F, E, self.down)
        # the next layer's first launch forms x2 = x1 + down while normalising; here it only delivers x2
        W.wsvd_rmsnorm_quant_i8(ctx, self.x1, self.down, self.g1, 1e-5, B, E, self.x2, self.tail_codes, self.tail_scale)


def _check_layer(c, L, gl, ref, before, what):
    sp, w = c.sp, c.w
    B = sp.batch
    assert W.wsvd_check(L.ctx) == 0
    assert (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    a, rmax, l2 = err_stats(gl.cq.cpu().numpy().astype(np.float64), ref["cQ"].reshape(B, -1))
    print(f"{what} c_Q: max_abs={a:.3e} rel_l2={l2:.3e}", flush=True)
    assert l2 <= 1e-3
    flips = _append_compare(L, c.cache, ref["cK"], ref["cV"], before, sp.latent_dtype)
    print(f"{what} store: boundary flips accepted = {flips}", flush=True)
    assert flips <= max(4, 2 * B * sp.n_kv_heads * sp.rank // 100)
    check_out(gl.u.cpu().numpy().astype(np.float64), ref["u"], sp.latent_dtype, f"{what} latent attention output")
    for key, got in (("x1", gl.x1), ("x2", gl.x2)):
        a, rmax, l2 = err_stats(got.cpu().numpy().astype(np.float64), ref[key].astype(np.float64))
        print(f"{what} {key}: max_abs={a:.3e} rel_l2={l2:.3e}", flush=True)
        # the GPU re-quantises its own intermediates four times on the way: codes on a rounding boundary may differ by
        # one step, which the bars of the integer paths cover
        assert a <= 2e-2 * max(1.0, np.abs(ref[key]).max()) and l2 <= 1e-3


@pytest.mark.parametrize("name,rq,F,over", [("c3_small", 32, 1408, dict()),
                                            ("c3_small", 32, 1408, dict(n_q_heads=8, n_kv_heads=4, context=700)),
                                            ("c5_small", 64, 1024, dict(n_q_heads=8, n_kv_heads=2)),
                                            ("c4_small", 32, 1408, dict()),
                                            ("c5_small", 64, 1024, dict())], ids=["i8", "i8g2", "i8r64g4", "i4", "i8r64g7"])
def test_decoder_layer_small(name, rq, F, over):
    c = build_layer_case(name, rq, F, **over)
    L = layer_for(c); L.upload(c.cache)
    before = c.cache.seq_lens.copy()
    ref = oracle_layer(c)
    gl = GpuLayer(c, L)
    gl.run(dev(c.x32), int(c.cache.seq_lens.max()))
    torch.cuda.synchronize()
    _check_layer(c, L, gl, ref, before, f"layer {name}")
    L.close()


def test_decoder_layer_full_size():
    """One layer at the batched int8 workload's shape (16 sequences, 32 heads, d_model 4096, rank 32, 2048 rows of
    context, FFN 11008), in the launch configuration the benchmark times."""
    c = build_layer_case("c3", 32, 11008, layer=1)
    L = layer_for(c); L.upload(c.cache)
    before = c.cache.seq_lens.copy()
    ref = oracle_layer(c)
    gl = GpuLayer(c, L)
    gl.run(dev(c.x32), int(c.cache.seq_lens.max()))
    torch.cuda.synchronize()
    _check_layer(c, L, gl, ref, before, "layer c3 full")
    L.close()
