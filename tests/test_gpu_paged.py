"""Paged cache: wsvd_latent_append_paged / wsvd_decode_attn_paged against the contiguous-cache entry points on the same
rows (bit-identical: the kernels do the same arithmetic, only the address of a tile or a row differs) and against the
oracle.  The pools are filled by scattering the pages of a contiguous device cache (pure byte moves, done with torch
indexing) through a shuffled block table, with more pages in the pool than the batch uses and poison in the rest."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
import wsvd_inputs as WI
from cases import build_case
from harness import as_dtype_dev, q_to_device
from test_gpu_parity import check_out, layer_for

pytestmark = pytest.mark.gpu


class Paged:
    """Pools + block table built from a DeviceLayer's contiguous planes."""

    def __init__(self, L, page_rows, seed=0, spare=5):
        self.L, self.P = L, page_rows
        assert L.t_cap % page_rows == 0
        self.max_pages = L.t_cap // page_rows
        self.n_pages = L.B * self.max_pages + spare
        rb = {"i8": L.r, "i4": L.r // 2}[L.latent_dtype]
        mb = {"i8": 2, "i4": 4}[L.latent_dtype]
        self.rb, self.mb = rb, mb
        cb, mbytes = W.wsvd_paged_cache_bytes(L.desc, page_rows, self.n_pages)
        assert cb == self.n_pages * L.Hkv * page_rows * rb and mbytes == self.n_pages * L.Hkv * page_rows * mb
        rng = np.random.default_rng(seed)
        perm = rng.permutation(self.n_pages)[: L.B * self.max_pages].reshape(L.B, self.max_pages)
        self.table_host = perm.astype(np.int32)
        self.table = torch.from_numpy(self.table_host).cuda()
        self.pools = [torch.full((self.n_pages, L.Hkv, page_rows * rb), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(2)]
        self.mpools = [torch.full((self.n_pages, L.Hkv, page_rows * mb), 0xFF, dtype=torch.uint8, device="cuda") for _ in range(2)]
        self.scatter()
        self.seq_lens = L.seq_lens.clone()
        self.cache = W.make_paged_cache(self.pools[0], self.pools[1], self.mpools[0], self.mpools[1], self.seq_lens, self.table,
                                        page_rows, self.max_pages, self.n_pages)

    def _views(self):
        L = self.L
        codes = [t.view(L.B, L.Hkv, self.max_pages, self.P * self.rb) for t in (L.k_codes, L.v_codes)]
        metas = [t[: L.B * L.Hkv * L.t_cap * self.mb].view(L.B, L.Hkv, self.max_pages, self.P * self.mb) for t in (L.k_meta, L.v_meta)]
        return codes, metas

    def scatter(self):
        codes, metas = self._views()
        idx = self.table.long().reshape(-1)
        for pl in range(2):
            self.pools[pl][idx] = codes[pl].permute(0, 2, 1, 3).reshape(-1, self.L.Hkv, self.P * self.rb)
            self.mpools[pl][idx] = metas[pl].permute(0, 2, 1, 3).reshape(-1, self.L.Hkv, self.P * self.mb)

    def gathered(self):
        """The pools' content in the shape of the contiguous planes."""
        L = self.L
        idx = self.table.long().reshape(-1)
        out = []
        for pl in range(2):
            c = self.pools[pl][idx].view(L.B, self.max_pages, L.Hkv, self.P * self.rb).permute(0, 2, 1, 3).reshape(-1)
            m = self.mpools[pl][idx].view(L.B, self.max_pages, L.Hkv, self.P * self.mb).permute(0, 2, 1, 3).reshape(-1)
            out.append((c, m))
        return out


CASES = [("c3_small", dict(), 64), ("c3_small", dict(context=1500, batch=2), 256), ("c4_small", dict(), 128),
         ("c3_small", dict(n_q_heads=8, n_kv_heads=2), 64), ("c5_small", dict(n_q_heads=4, n_kv_heads=2), 64),
         # 5..8 query heads per kv head: head sets of 4 in consecutive launches (int8: the contiguous cache runs another kernel)
         ("c5_small", dict(), 64), ("c3_small", dict(n_q_heads=10, n_kv_heads=2, context=1500, batch=2), 256),
         ("c4_small", dict(n_q_heads=24, n_kv_heads=4), 128)]


@pytest.mark.parametrize("name,over,page_rows", CASES, ids=["i8", "i8-split-context", "i4-ragged", "i8-4-heads-per-kv", "i8-rank64",
                                                            "i8-rank64-7-heads-per-kv", "i8-5-heads-per-kv-split-context", "i4-6-heads-per-kv"])
def test_paged_attention_and_append_equal_the_contiguous_ones(name, over, page_rows):
    c = build_case(name, **over)
    sp = c.sp
    t_cap = (c.t_cap + page_rows - 1) // page_rows * page_rows
    L = layer_for(c, t_cap=t_cap); L.upload(c.cache)
    PG = Paged(L, page_rows, seed=len(name) + page_rows)
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    n_max = int(c.cache.seq_lens.max())
    # int8 latents with more than 4 query heads per kv head: the contiguous cache goes through the grouped-query kernel,
    # the paged one through the paired-block kernel; equal up to rounding, not bit for bit
    same_kernel = not (sp.latent_dtype == "i8" and sp.n_q_heads // sp.n_kv_heads > 4)
    # ---- attention over the uploaded rows
    want = L.attend(qd, qs, BKd, BVd, n_max)
    out = torch.full_like(L.out, float("nan"))
    W.wsvd_decode_attn_paged(L.ctx, L.desc, qd, qs, BKd, BVd, PG.cache, n_max, out)
    assert W.wsvd_check(L.ctx) == 0
    got = out.cpu().numpy().astype(np.float64)
    assert (got == want).all() or not same_kernel, "paged attention differs from the contiguous one"
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()
    ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    check_out(got, ref, sp.latent_dtype, f"paged attention {name}")
    # ---- three appends on both caches (rows cross page and tile boundaries in the ragged cases), then attention again
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    for step in range(3):
        x = WI.bf16_exact(WI.hidden_states(sp, sp.batch, 1.0, which="new", sub=50 + step))
        xd = as_dtype_dev(x, "bf16")
        O.latent_append(c.cache, x.astype(np.float64), c.AK.astype(np.float64), c.AV.astype(np.float64))
        assert L.append(xd, None, AKd, AVd) == 0
        W.wsvd_latent_append_paged(L.ctx, L.desc, xd, None, AKd, AVd, PG.cache)
        assert W.wsvd_check(L.ctx) == 0
    assert (PG.seq_lens.cpu().numpy() == c.cache.seq_lens).all() and (L.seq_lens.cpu().numpy() == c.cache.seq_lens).all()
    rb, mb = PG.rb, PG.mb
    planes = [(L.k_codes, L.k_meta), (L.v_codes, L.v_meta)]
    for pl, (gc, gm) in enumerate(PG.gathered()):
        wc = planes[pl][0].view(sp.batch, sp.n_kv_heads, t_cap, -1) if sp.latent_dtype == "i8" else None
        a = gc.view(sp.batch, sp.n_kv_heads, -1).cpu().numpy(); b = planes[pl][0].view(sp.batch, sp.n_kv_heads, -1).cpu().numpy()
        am = gm.view(sp.batch, sp.n_kv_heads, -1).cpu().numpy()
        bm = planes[pl][1][: sp.batch * sp.n_kv_heads * t_cap * mb].view(sp.batch, sp.n_kv_heads, -1).cpu().numpy()
        for bi in range(sp.batch):
            # whole 64-row blocks below the sequence's length hold the same bytes in both caches (rows past it are poison
            # in both, but int4 value bytes pair two rows: compare up to the last complete pair)
            n = int(c.cache.seq_lens[bi])
            n_cmp = n // 64 * 64
            assert a[bi, :, : n_cmp * rb].tobytes() == b[bi, :, : n_cmp * rb].tobytes(), (name, pl, bi)
            assert am[bi, :, : n * mb].tobytes() == bm[bi, :, : n * mb].tobytes(), (name, pl, bi)
    n_max = int(c.cache.seq_lens.max())
    want = L.attend(qd, qs, BKd, BVd, n_max)
    out.fill_(float("nan"))
    W.wsvd_decode_attn_paged(L.ctx, L.desc, qd, qs, BKd, BVd, PG.cache, n_max, out)
    assert W.wsvd_check(L.ctx) == 0
    got = out.cpu().numpy().astype(np.float64)
    assert (got == want).all() or not same_kernel, "paged attention after paged appends differs from the contiguous path"
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()
    ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    check_out(got, ref, sp.latent_dtype, f"paged append + attention {name}")
    L.close()


def test_paged_cache_argument_checks_and_bad_entries():
    c = build_case("c3_small")
    sp = c.sp
    L = layer_for(c, t_cap=384); L.upload(c.cache)
    PG = Paged(L, 64)
    qd, qs, _ = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    out = torch.full_like(L.out, float("nan"))
    bad = W.make_paged_cache(PG.pools[0], PG.pools[1], PG.mpools[0], PG.mpools[1], PG.seq_lens, PG.table, 64, PG.max_pages + 1, PG.n_pages)
    with pytest.raises(W.WsvdError) as e:            # max_pages * page_rows must be the descriptor's t_cap
        W.wsvd_decode_attn_paged(L.ctx, L.desc, qd, qs, BKd, BVd, bad, 333, out)
    assert e.value.status == W.E_SHAPE
    bad = W.make_paged_cache(PG.pools[0], PG.pools[1], PG.mpools[0], PG.mpools[1], PG.seq_lens, PG.table, 96, 4, PG.n_pages)
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_decode_attn_paged(L.ctx, L.desc, qd, qs, BKd, BVd, bad, 333, out)
    assert e.value.status == W.E_SHAPE
    assert torch.isnan(out).all()
    # an append into a row whose table entry is outside the pools: nothing stored, reported, the other sequences go through
    tbl = PG.table.clone()
    page_of_new_row = int(c.cache.seq_lens[1]) // 64
    tbl[1, page_of_new_row] = PG.n_pages + 7
    before = [p.clone() for p in PG.pools]
    broken = W.make_paged_cache(PG.pools[0], PG.pools[1], PG.mpools[0], PG.mpools[1], PG.seq_lens, tbl, 64, PG.max_pages, PG.n_pages)
    x = WI.bf16_exact(c.x_new[0])
    W.wsvd_latent_append_paged(L.ctx, L.desc, as_dtype_dev(x, "bf16"), None, L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16"), broken)
    assert W.wsvd_check(L.ctx) == W.E_SHAPE
    touched = [(a != b).flatten(1).any(1).nonzero().flatten().tolist() for a, b in zip(PG.pools, before)]
    good_pages = {int(PG.table_host[b, int(c.cache.seq_lens[b]) // 64]) for b in range(sp.batch) if b != 1}
    assert set(touched[0]) <= good_pages and set(touched[1]) <= good_pages and len(touched[0]) > 0
    L.close()


@pytest.mark.parametrize("name,over,all_seqs", [("c3_small", dict(), False), ("c3_small", dict(), True),
                                                ("c5_small", dict(n_q_heads=4, n_kv_heads=2), False), ("c4_small", dict(batch=4, context=300, ragged=(100, 300)), False),
                                                ("c4_small", dict(batch=4, context=300, ragged=(100, 300)), True)],
                         ids=["i8-one", "i8-all", "i8-rank64-one", "i4-one", "i4-all"])
def test_paged_prefill_equals_the_contiguous_one(name, over, all_seqs):
    """wsvd_prefill_append_paged against wsvd_prefill_append (the same tiled projection, only the address of a row
    differs): the same bytes in the pages as in the contiguous planes, the same attention afterwards; a prompt that
    crosses several pages; a table entry outside the pools."""
    c = build_case(name, extra_cap=300, **over)
    sp = c.sp
    if sp.latent_dtype == "i4":
        c.cache.seq_lens[:] = c.cache.seq_lens // 2 * 2       # the tiled int4 store wants an even start row
    L = layer_for(c); L.upload(c.cache)
    PG = Paged(L, 64, seed=11)
    n = 70 if all_seqs else (150 if sp.latent_dtype == "i4" else 151)     # (int4: the next block starts on an even row again)
    AKd, AVd = L.pack_A(c.AK, "bf16"), L.pack_A(c.AV, "bf16")
    lens0 = c.cache.seq_lens.copy()
    if all_seqs:
        X = np.stack([WI.bf16_exact(WI.hidden_states(sp, n, 1.0, which="ctx", sub=60 + b)) for b in range(sp.batch)])
        xd, seq, targets = as_dtype_dev(X.reshape(sp.batch * n, -1), "bf16"), -1, list(range(sp.batch))
    else:
        b = 1
        xd, seq, targets = as_dtype_dev(WI.bf16_exact(WI.hidden_states(sp, n, 1.0, which="ctx", sub=77)), "bf16"), b, [b]
    W.wsvd_prefill_append(L.ctx, L.desc, xd, None, n, seq, AKd, AVd, L.cache)
    assert W.wsvd_check(L.ctx) == 0
    W.wsvd_prefill_append_paged(L.ctx, L.desc, xd, n, seq, AKd, AVd, PG.cache)
    assert W.wsvd_check(L.ctx) == 0
    want_lens = lens0 + np.array([n if b in targets else 0 for b in range(sp.batch)])
    assert (PG.seq_lens.cpu().numpy() == want_lens).all() and (L.seq_lens.cpu().numpy() == want_lens).all()
    rb, mb = PG.rb, PG.mb
    planes = [(L.k_codes, L.k_meta), (L.v_codes, L.v_meta)]
    t_cap = L.t_cap
    for pl, (gc, gm) in enumerate(PG.gathered()):
        a = gc.view(sp.batch, sp.n_kv_heads, -1).cpu().numpy(); bb = planes[pl][0].view(sp.batch, sp.n_kv_heads, -1).cpu().numpy()
        am = gm.view(sp.batch, sp.n_kv_heads, -1).cpu().numpy()
        bm = planes[pl][1][: sp.batch * sp.n_kv_heads * t_cap * mb].view(sp.batch, sp.n_kv_heads, -1).cpu().numpy()
        for bi in range(sp.batch):
            nn = int(want_lens[bi])
            n_cmp = nn // 64 * 64
            assert a[bi, :, : n_cmp * rb].tobytes() == bb[bi, :, : n_cmp * rb].tobytes(), (name, pl, bi)
            assert am[bi, :, : nn * mb].tobytes() == bm[bi, :, : nn * mb].tobytes(), (name, pl, bi)
    qd, qs, _ = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    n_max = int(want_lens.max())
    want = L.attend(qd, qs, BKd, BVd, n_max)
    out = torch.full_like(L.out, float("nan"))
    W.wsvd_decode_attn_paged(L.ctx, L.desc, qd, qs, BKd, BVd, PG.cache, n_max, out)
    assert W.wsvd_check(L.ctx) == 0
    assert (out.cpu().numpy().astype(np.float64) == want).all(), "attention over the paged prompt differs from the contiguous one"
    # a table entry outside the pools under the rows of a second prompt block: reported, those rows not stored
    tbl = PG.table.clone()
    tb = targets[0]
    bad_page = int(want_lens[tb]) // 64 + 1                    # the page after the one the block starts in
    tbl[tb, bad_page] = PG.n_pages + 3
    before = [p.clone() for p in PG.pools]
    broken = W.make_paged_cache(PG.pools[0], PG.pools[1], PG.mpools[0], PG.mpools[1], PG.seq_lens, tbl, 64, PG.max_pages, PG.n_pages)
    n2 = 130
    x2 = as_dtype_dev(WI.bf16_exact(WI.hidden_states(sp, n2, 1.0, which="ctx", sub=99)), "bf16")
    W.wsvd_prefill_append_paged(L.ctx, L.desc, x2, n2, tb, AKd, AVd, broken)
    assert W.wsvd_check(L.ctx) == W.E_SHAPE
    touched = set((PG.pools[0] != before[0]).flatten(1).any(1).nonzero().flatten().tolist())
    first = int(want_lens[tb]) // 64
    allowed = {int(PG.table_host[tb, pg]) for pg in range(first, min(PG.max_pages, (int(want_lens[tb]) + n2 + 63) // 64)) if pg != bad_page}
    assert touched and touched <= allowed, (touched, allowed)
    L.close()


@pytest.mark.parametrize("name,over,nq,n_after", [("c3_small", dict(context=500, ragged=(20, 500), batch=4), 70, 0),
                                                  ("c3_small", dict(n_q_heads=8, n_kv_heads=4, context=300), 33, 5),
                                                  ("c5_small", dict(n_q_heads=4, n_kv_heads=2, context=400), 40, 0)],
                         ids=["i8", "i8-2-heads-per-kv-later-rows", "i8-rank64"])
def test_paged_prompt_attention_equals_the_contiguous_one(name, over, nq, n_after):
    """wsvd_prefill_attn_paged against wsvd_prefill_attn's tiled kernel on the same rows (pages of 64 rows in shuffled
    order, poison in the spare ones): bit-identical, and close to the oracle."""
    c = build_case(name, **over)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    PG = Paged(L, 64, seed=5)
    G = sp.n_q_heads // sp.n_kv_heads
    rng = np.random.default_rng(9)
    q32 = WI.bf16_exact(rng.standard_normal((sp.batch, sp.n_kv_heads, nq, G, sp.d_head)).astype(np.float32))
    d = type(L.desc).from_buffer_copy(L.desc)
    d.q_dtype = W.DTYPES["bf16"]
    qd = as_dtype_dev(q32, "bf16")
    BKd, BVd = as_dtype_dev(c.BK, "bf16"), as_dtype_dev(c.BV, "bf16")
    n_max = int(c.cache.seq_lens.max())
    want = torch.full(q32.shape, float("nan"), dtype=torch.float32, device="cuda")
    W.wsvd_prefill_attn(L.ctx, d, qd, nq, n_after, BKd, BVd, L.cache, n_max, want)
    got = torch.full(q32.shape, float("nan"), dtype=torch.float32, device="cuda")
    W.wsvd_prefill_attn_paged(L.ctx, d, qd, nq, n_after, BKd, BVd, PG.cache, n_max, got)
    assert W.wsvd_check(L.ctx) == 0
    assert (got.cpu().view(torch.int32) == want.cpu().view(torch.int32)).all()
    ref = O.causal_attn_reconstructed(c.cache, q32.astype(np.float64), c.BK.astype(np.float64), c.BV.astype(np.float64),
                                      c.sm_scale, n_after=n_after)
    check_out(got.cpu().numpy().astype(np.float64), ref, "i8", f"paged prompt attention {name}")
    L.close()
