"""HIP-graph replays of the hot calls against the same calls launched eagerly.

A serving loop captures the decode step once and replays it; the sequence lengths live on the device and advance with
every replay, so one captured graph serves consecutive steps.  Every replay is compared bit for bit with the eager run
of the same step (all kernels here are deterministic: partial results are always combined in a fixed order), with the
program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
import wsvd_inputs as WI
from cases import build_case
from harness import as_dtype_dev, dev, q_to_device
from test_gpu_layer import GpuLayer, build_layer_case
from test_gpu_parity import layer_for

pytestmark = pytest.mark.gpu

N_STEPS = 4


def _snapshot(L):
    return [t.clone() for t in (L.k_codes, L.v_codes, L.k_meta, L.v_meta, L.seq_lens)]


def _restore(L, snap):
    for t, s in zip((L.k_codes, L.v_codes, L.k_meta, L.v_meta, L.seq_lens), snap):
        t.copy_(s)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["c3_small", "c4_small", "c2_small"])
def test_decode_step_graph_replays_equal_eager(name):
    """append + attention captured once, replayed for consecutive tokens of the same sequences."""
    c = build_case(name)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    xdt = "f32" if sp.factor_dtype == "f32" else "bf16"
    x = as_dtype_dev(WI.bf16_exact(c.x_new[0]) if xdt == "bf16" else c.x_new[0], xdt)
    AKd, AVd = L.pack_A(c.AK, sp.factor_dtype), L.pack_A(c.AV, sp.factor_dtype)
    BKd, BVd = as_dtype_dev(c.BK, sp.factor_dtype), as_dtype_dev(c.BV, sp.factor_dtype)
    qd, qs, _ = q_to_device(c.q32[0], sp.q_dtype)
    max_len = int(c.cache.seq_lens.max()) + N_STEPS
    snap = _snapshot(L)

    def step():
        W.wsvd_latent_append(L.ctx, L.desc, x, None, AKd, AVd, L.cache)
        W.wsvd_decode_attn(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, max_len, L.out)

    eager = []
    for _ in range(N_STEPS):
        step()
        torch.cuda.synchronize()
        eager.append(L.out.cpu().numpy().copy())
    assert W.wsvd_check(L.ctx) == 0
    lens_after = L.seq_lens.cpu().numpy().copy()
    assert not np.array_equal(eager[0], eager[-1]), "consecutive steps must differ (the cache grows)"

    _restore(L, snap)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()                                    # warm-up on the capture stream (not part of the comparison) ...
        stream.synchronize()
    _restore(L, snap)                             # ... undone
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(g, stream=stream):
            step()
    _restore(L, snap)                             # capture does not execute, but make the starting state explicit
    scratch = torch.zeros(1 << 16, device="cuda")
    for i in range(N_STEPS):
        g.replay()
        torch.cuda.synchronize()
        got = L.out.cpu().numpy()
        assert np.array_equal(got, eager[i]), f"replay {i} differs from the eager step {i}"
        scratch.add_(1.0)                         # unrelated eager work between replays
        assert float(scratch.sum()) == (i + 1) * scratch.numel()
    assert W.wsvd_check(L.ctx) == 0
    assert (L.seq_lens.cpu().numpy() == lens_after).all()
    L.close()


def test_decoder_layer_graph_replays_equal_eager():
    """The ten launches of a quantised decoder layer, captured once and replayed for consecutive tokens."""
    c = build_layer_case("c3_small", 32, 1408)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    gl = GpuLayer(c, L)
    x = dev(c.x32)
    max_len = int(c.cache.seq_lens.max()) + N_STEPS
    torch.cuda.synchronize()
    snap = _snapshot(L)
    eager = []
    for _ in range(N_STEPS):
        gl.run(x, max_len)
        torch.cuda.synchronize()
        eager.append((gl.x2.cpu().numpy().copy(), gl.u.cpu().numpy().copy()))
    assert W.wsvd_check(L.ctx) == 0
    assert not np.array_equal(eager[0][1], eager[-1][1])

    _restore(L, snap)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        gl.run(x, max_len)
        stream.synchronize()
    _restore(L, snap)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(g, stream=stream):
            gl.run(x, max_len)
    _restore(L, snap)
    for i in range(N_STEPS):
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(gl.u.cpu().numpy(), eager[i][1]), f"replay {i}: attention output differs from the eager step"
        assert np.array_equal(gl.x2.cpu().numpy(), eager[i][0]), f"replay {i}: layer output differs from the eager step"
        _ = torch.randn(1024, device="cuda").sum().item()      # unrelated eager work and a synchronisation in between
    assert W.wsvd_check(L.ctx) == 0
    L.close()


def test_rotary_attention_graph_replays_equal_eager():
    c = build_case("c3_small", context=700)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    qd, qs, _ = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    n = int(c.cache.seq_lens.max())
    W.wsvd_decode_attn_rope(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, n, 10000.0, L.out)
    torch.cuda.synchronize()
    ref = L.out.cpu().numpy().copy()
    stream = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(g, stream=stream):
            W.wsvd_decode_attn_rope(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, n, 10000.0, L.out)
    for i in range(3):
        L.out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(L.out.cpu().numpy(), ref), f"rotary replay {i}"
    assert W.wsvd_check(L.ctx) == 0
    L.close()


def test_prefill_graph_replays_equal_eager():
    """The two prompt-sized launches (tiled projection of all sequences, tiled causal attention) captured once; every
    replay starts from the same lengths (a fill kernel inside the graph resets them) and must reproduce the eager
    cache and outputs bit for bit."""
    c = build_case("c3_small", extra_cap=256)
    sp = c.sp
    G = sp.n_q_heads // sp.n_kv_heads
    L = layer_for(c); L.upload(c.cache)
    n = 150
    X = np.stack([WI.bf16_exact(WI.hidden_states(sp, n, 1.0, which="ctx", sub=60 + b)) for b in range(sp.batch)])
    xd = as_dtype_dev(X.reshape(sp.batch * n, -1), "bf16")
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    rng = np.random.default_rng(21)
    q = as_dtype_dev(WI.bf16_exact(rng.standard_normal((sp.batch, sp.n_kv_heads, n, G, sp.d_head)).astype(np.float32)), "bf16")
    out = torch.empty((sp.batch, sp.n_kv_heads, n, G, sp.d_head), dtype=torch.float32, device="cuda")
    d = type(L.desc).from_buffer_copy(L.desc); d.q_dtype = W.DTYPES["bf16"]
    lens0 = L.seq_lens.clone()
    torch.cuda.synchronize()
    snap = _snapshot(L)

    def step():
        L.seq_lens.copy_(lens0)                   # a copy kernel, not a memset node
        W.wsvd_prefill_append(L.ctx, L.desc, xd, None, n, -1, AKd, AVd, L.cache)
        W.wsvd_prefill_attn(L.ctx, d, q, n, 0, BKd, BVd, L.cache, int(c.cache.seq_lens.max()) + n, out)

    step(); torch.cuda.synchronize()
    assert W.wsvd_check(L.ctx) == 0
    ref_out = out.cpu().numpy().copy()
    ref = _snapshot(L)
    assert (ref[4].cpu().numpy() == lens0.cpu().numpy() + n).all()
    _restore(L, snap)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step(); stream.synchronize()
    _restore(L, snap)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(g, stream=stream):
            step()
    for i in range(3):
        _restore(L, snap)                         # the cache as it was before the prompt
        out.fill_(float("nan")); torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref_out), f"prefill replay {i}: attention output differs"
        for t, r in zip((L.k_codes, L.v_codes, L.k_meta, L.v_meta, L.seq_lens), ref):
            assert torch.equal(t, r), f"prefill replay {i}: cache differs"
        _ = torch.randn(2048, device="cuda").sum().item()
    assert W.wsvd_check(L.ctx) == 0
    L.close()


def test_shared_latent_graph_replays_equal_eager():
    from test_gpu_shared import SharedCase, H
    c = SharedCase(3, 512, 128, [700, 130, 0], 768)
    ctx = W.wsvd_create(0)
    kc, vc, ks, vs, sl = c.device()
    ws = torch.empty(W.wsvd_shared_workspace_bytes(c.B, H, c.d, c.R, c.t_cap), dtype=torch.uint8, device="cuda")
    out = torch.empty((c.B, H, c.d), dtype=torch.float32, device="cuda")
    q, BK, BV = as_dtype_dev(c.q, "bf16"), as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")

    def step():
        W.wsvd_decode_attn_shared(ctx, c.B, H, c.d, c.R, c.t_cap, c.sm, q, BK, BV, kc, vc, ks, vs, sl, ws, out)

    step(); torch.cuda.synchronize()
    ref = out.cpu().numpy().copy()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step(); stream.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(g, stream=stream):
            step()
    for i in range(3):
        out.fill_(float("nan")); ws.fill_(0xFF); torch.cuda.synchronize()      # stale workspace contents must not matter
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref), f"shared-latent replay {i}"
        _ = torch.randn(2048, device="cuda").sum().item()
    assert W.wsvd_check(ctx) == 0
    W.wsvd_destroy(ctx)
