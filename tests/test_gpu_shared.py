"""GPU parity tests of the shared-latent ("whole-matrix") decode attention, the scheme the per-head method is contrasted
with: wsvd_decode_attn_shared against the oracle's decode_attn_shared_latent on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
import wsvd_inputs as WI
from harness import as_dtype_dev
from test_gpu_parity import check_out

pytestmark = pytest.mark.gpu

H = 32


def k_image(codes):
    """[T, R] int8 -> the K plane's byte order: 32-token blocks; per block [R/32][dim half][token][16 dims]."""
    T, R = codes.shape
    return np.ascontiguousarray(codes.reshape(T // 32, 32, R // 32, 2, 16).transpose(0, 2, 3, 1, 4)).reshape(-1)


def v_image(codes):
    """[T, R] int8 -> the V plane's byte order: 32-token blocks; per block [R/32][token half][dim][16 tokens]."""
    T, R = codes.shape
    return np.ascontiguousarray(codes.reshape(T // 32, 2, 16, R // 32, 32).transpose(0, 3, 1, 4, 2)).reshape(-1)


class SharedCase:
    def __init__(self, batch, R, d, lens, t_cap, seed_name="c3_small", garbage=True):
        self.sp = sp = WI.spec(seed_name, batch=batch, d_head=d, n_q_heads=H, n_kv_heads=H)
        self.B, self.R, self.d, self.t_cap = batch, R, d, t_cap
        self.sm = d ** -0.5
        self.cache = O.LatentCache(batch, 1, t_cap, R, "i8")
        g = np.random.default_rng(1234)
        if garbage:      # rows past a sequence's end hold anything: random codes, NaN scales
            self.cache.k[:] = g.integers(-128, 128, self.cache.k.shape, dtype=np.int8)
            self.cache.v[:] = g.integers(-128, 128, self.cache.v.shape, dtype=np.int8)
            self.cache.k_scale[:] = np.float16(np.nan); self.cache.v_scale[:] = np.float16(np.nan)
        for b, n in enumerate(lens):
            if n:
                self.cache.store_rows("k", b, 0, WI.shared_latents(sp, R, "k", b, n).astype(np.float64)[None])
                self.cache.store_rows("v", b, 0, WI.shared_latents(sp, R, "v", b, n).astype(np.float64)[None])
            self.cache.seq_lens[b] = n
        self.BK, self.BV = WI.shared_up_factors(sp, R)
        self.q = WI.bf16_exact(WI.normal(sp.seed, 77, (batch, H, d)))

    def device(self):
        c = self.cache
        kc = torch.from_numpy(np.stack([k_image(c.k[b, 0]) for b in range(self.B)]).view(np.uint8)).cuda()
        vc = torch.from_numpy(np.stack([v_image(c.v[b, 0]) for b in range(self.B)]).view(np.uint8)).cuda()
        ks = torch.from_numpy(np.ascontiguousarray(c.k_scale[:, 0]).view(np.int16)).cuda()
        vs = torch.from_numpy(np.ascontiguousarray(c.v_scale[:, 0]).view(np.int16)).cuda()
        sl = torch.from_numpy(c.seq_lens.astype(np.int32)).cuda()
        return kc, vc, ks, vs, sl

    def run(self, ctx):
        kc, vc, ks, vs, sl = self.device()
        # the entry point takes plain pointers: make sure every buffer has the size its arguments promise
        assert self.BK.shape == (H, self.R, self.d) and self.BV.shape == (H, self.R, self.d) and self.q.shape == (self.B, H, self.d)
        assert kc.numel() == self.B * self.t_cap * self.R == vc.numel() and ks.numel() == self.B * self.t_cap == vs.numel()
        assert sl.numel() == self.B
        ws = torch.empty(W.wsvd_shared_workspace_bytes(self.B, H, self.d, self.R, self.t_cap), dtype=torch.uint8, device="cuda")
        out = torch.full((self.B, H, self.d), float("nan"), dtype=torch.float32, device="cuda")
        W.wsvd_decode_attn_shared(ctx, self.B, H, self.d, self.R, self.t_cap, self.sm, as_dtype_dev(self.q, "bf16"),
                                  as_dtype_dev(self.BK, "bf16"), as_dtype_dev(self.BV, "bf16"), kc, vc, ks, vs, sl, ws, out)
        torch.cuda.synchronize()
        assert W.wsvd_check(ctx) == 0
        return out.cpu().numpy().astype(np.float64)

    def oracle(self, heads=None):
        return O.decode_attn_shared_latent(self.cache, self.q.astype(np.float64), self.BK.astype(np.float64),
                                           self.BV.astype(np.float64), self.sm, heads=heads)


CASES = [
    ("r256", 2, 256, 128, [300, 129], 384),
    ("r512-d64", 3, 512, 64, [1, 128, 513], 640),
    ("r1024-empty", 2, 1024, 128, [700, 0], 768),
    ("r256-long", 1, 256, 128, [4000], 4096),           # several chunks per split
    ("r1024-batch40", 40, 1024, 64, [130 + 7 * b for b in range(40)], 512),
    # ranks above 1024: the latent walked in slabs of 1024 dims (the last slab of 3712 has 640, that of 1152 has 128)
    ("r2048", 2, 2048, 128, [300, 129], 384),
    ("r3712-ragged", 3, 3712, 128, [1, 515, 1000], 1024),
    ("r2560-d64-long", 1, 2560, 64, [4000], 4096),
    ("r1280-3-chunks-per-split", 40, 1280, 64, [2000 - 47 * b for b in range(40)], 2048),
    ("r1152-4-chunks-per-split", 64, 1152, 64, [2048 - 30 * b for b in range(64)], 2048),
]


@pytest.mark.parametrize("name,batch,R,d,lens,t_cap", CASES, ids=[c[0] for c in CASES])
def test_shared_latent_attention_matches_oracle(name, batch, R, d, lens, t_cap):
    print(f"shared-latent case {name}: B={batch} R={R} d={d} t_cap={t_cap}", flush=True)
    c = SharedCase(batch, R, d, lens, t_cap)
    ctx = W.wsvd_create(0)
    got = c.run(ctx)
    ref = c.oracle()
    for b, n in enumerate(lens):
        if n == 0:
            assert (got[b] == 0).all()
    check_out(got, ref, "i8", f"shared latent {name}")
    W.wsvd_destroy(ctx)


def test_shared_latent_full_size_sampled():
    """The contrast workload of the benchmark: 16 sequences x 2048 tokens, one shared latent of rank 1024 (the cache
    bytes of 32 heads x rank 32); the oracle computes a sample of (sequence, head) pairs."""
    B, R, d, T = 16, 1024, 128, 2048
    print("shared-latent full size: building the oracle cache", flush=True)
    c = SharedCase(B, R, d, [T] * B, T, seed_name="c3", garbage=False)
    ctx = W.wsvd_create(0)
    print("shared-latent full size: GPU call", flush=True)
    got = c.run(ctx)
    rng = np.random.default_rng(3)
    heads = [(int(b), int(h)) for b, h in zip(rng.integers(0, B, 20), rng.integers(0, H, 20))] + [(0, 0), (B - 1, H - 1)]
    ref = c.oracle(heads=heads)
    assert np.isfinite(got).all()
    check_out(got, ref, "i8", f"shared latent, full size, {len(heads)} sampled (sequence, head) pairs")
    W.wsvd_destroy(ctx)


def test_shared_latent_sweep_rank_full_size_sampled():
    """The widest rank of the rank sweep (32 heads x per-head rank 115 = 3680, run as 3712) at 16 sequences x 2048 tokens."""
    B, R, d, T = 16, 3712, 128, 2048
    print("shared-latent rank 3712: building the oracle cache", flush=True)
    c = SharedCase(B, R, d, [T] * B, T, seed_name="c3", garbage=False)
    ctx = W.wsvd_create(0)
    print("shared-latent rank 3712: GPU call", flush=True)
    got = c.run(ctx)
    rng = np.random.default_rng(4)
    heads = [(int(b), int(h)) for b, h in zip(rng.integers(0, B, 8), rng.integers(0, H, 8))] + [(0, 0), (B - 1, H - 1)]
    ref = c.oracle(heads=heads)
    assert np.isfinite(got).all()
    check_out(got, ref, "i8", f"shared latent rank 3712, full size, {len(heads)} sampled (sequence, head) pairs")
    W.wsvd_destroy(ctx)


def test_shared_latent_argument_errors():
    c = SharedCase(1, 256, 128, [40], 128)
    ctx = W.wsvd_create(0)
    kc, vc, ks, vs, sl = c.device()
    q, BK, BV = as_dtype_dev(c.q, "bf16"), as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    ws = torch.empty(W.wsvd_shared_workspace_bytes(1, H, 128, 256, 128), dtype=torch.uint8, device="cuda")
    out = torch.empty((1, H, 128), dtype=torch.float32, device="cuda")

    def call(batch=1, heads=H, d=128, R=256, t_cap=128, wsp=ws):
        W.wsvd_decode_attn_shared(ctx, batch, heads, d, R, t_cap, 0.0, q, BK, BV, kc, vc, ks, vs, sl, wsp, out)

    for kw, status in ((dict(heads=16), W.E_UNSUPPORTED), (dict(R=128), W.E_UNSUPPORTED), (dict(R=1100), W.E_UNSUPPORTED),
                       (dict(R=4224), W.E_UNSUPPORTED), (dict(t_cap=100), W.E_SHAPE),
                       (dict(d=96), W.E_SHAPE), (dict(batch=0), W.E_SHAPE), (dict(wsp=ws[:1024]), W.E_WORKSPACE)):
        with pytest.raises(W.WsvdError) as e:
            call(**kw)
        assert e.value.status == status, kw
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_shared_workspace_bytes(1, 8, 128, 256, 128)
    assert e.value.status == W.E_UNSUPPORTED
    call()                                          # sm_scale <= 0: 1 / sqrt(d)
    torch.cuda.synchronize()
    check_out(out.cpu().numpy().astype(np.float64), c.oracle(), "i8", "shared latent, default scale")
    W.wsvd_destroy(ctx)
