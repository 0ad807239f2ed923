"""The allocation-free variant of the decode attention (wsvd_decode_attn_static: split partials and tickets in a static
device array of the library instead of a caller's workspace) against wsvd_decode_attn, through the C ABI: two calls in
a row, the second with a smaller input, each bit-identical to the existing entry point and within the bars against
the oracle.  Collected last so that a failure here cannot hide another test's."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2604_02570_amd as W
from cases import build_case
from harness import as_dtype_dev, q_to_device
from test_gpu_parity import check_out, layer_for

pytestmark = pytest.mark.gpu


def _both(c):
    """(output of wsvd_decode_attn, output of wsvd_decode_attn_static, oracle) for a case; the layer's context HAS a
    workspace for the first call; the static call gets a context of its own that never saw one."""
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    qd, qs, q64 = q_to_device(c.q32[0], sp.q_dtype)
    fd = sp.factor_dtype
    BKd, BVd = as_dtype_dev(c.BK, fd), as_dtype_dev(c.BV, fd)
    n_max = int(c.cache.seq_lens.max())
    want = L.attend(qd, qs, BKd, BVd, n_max)
    bare = W.wsvd_create(0)                       # no wsvd_set_workspace on this one
    W.wsvd_ctx_set_option(bare, "min_chunk", 256)  # the layer's decomposition: bit-equal outputs, and splits in use
    out = torch.full_like(L.out, float("nan"))
    W.wsvd_decode_attn_static(bare, L.desc, qd, qs, BKd, BVd, L.cache, n_max, out)
    assert W.wsvd_check(bare) == 0
    got = out.cpu().numpy().astype(np.float64)
    ref = O.decode_attn_reconstructed(c.cache, q64, c.BK.astype(np.float64), c.BV.astype(np.float64), c.sm_scale)
    W.wsvd_destroy(bare)
    L.close()
    return want, got, ref


def test_static_scratch_attention_matches_the_workspace_one():
    # 1. a context that is split over several workgroups, so that partials and tickets are in use
    big = build_case("c3_small", context=2000, batch=2)
    want, got, ref = _both(big)
    assert (got == want).all(), "static-scratch call differs from wsvd_decode_attn"
    check_out(got, ref, "i8", "static scratch, 2 x 2000 rows")
    # 2. right after it a smaller input (fewer sequences, shorter, ragged int4): stale partials of call 1 lie around
    small = build_case("c4_small", batch=3, context=700, ragged=(300, 700))
    want, got, ref = _both(small)
    assert (got == want).all(), "second, smaller static-scratch call differs from wsvd_decode_attn"
    check_out(got, ref, "i4", "static scratch, smaller second call")
    # 3. fp32 latents take the same route (vector-ALU kernel)
    c1 = build_case("c1", batch=2, context=1500)
    want, got, ref = _both(c1)
    assert (got == want).all()
    check_out(got, ref, "f32", "static scratch, fp32 latents")


def test_static_scratch_rejects_what_does_not_fit():
    """The split words a launch needs are bounded by what the chip runs at a time (a few MB at most with the default launch
    policy), so the rejection is shown by shrinking the limit: the call below is valid in every other respect (all its
    buffers have the sizes the descriptor promises), it is just not allowed the 300 KB of words its two splits need."""
    c = build_case("c3_small", context=2000, batch=2)
    sp = c.sp
    L = layer_for(c); L.upload(c.cache)
    qd, qs, _ = q_to_device(c.q32[0], sp.q_dtype)
    BKd, BVd = as_dtype_dev(c.BK, sp.factor_dtype), as_dtype_dev(c.BV, sp.factor_dtype)
    n_max = int(c.cache.seq_lens.max())
    out = torch.full_like(L.out, float("nan"))
    W.wsvd_ctx_set_option(L.ctx, "static_limit_kib", 65)           # counters (64 KiB) + 1 KiB
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_decode_attn_static(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, n_max, out)
    assert e.value.status == W.E_WORKSPACE
    assert torch.isnan(out).all(), "a rejected call must not enqueue anything"
    W.wsvd_ctx_set_option(L.ctx, "static_limit_kib", 0)
    W.wsvd_decode_attn_static(L.ctx, L.desc, qd, qs, BKd, BVd, L.cache, n_max, out)     # the same call fits the real array
    assert W.wsvd_check(L.ctx) == 0 and torch.isfinite(out).all()
    with pytest.raises(W.WsvdError) as e:         # the other host-side checks are wsvd_decode_attn's
        W.wsvd_decode_attn_static(L.ctx, L.desc, qd, None, BKd, BVd, L.cache, n_max, out)
    assert e.value.status == W.E_NULL
    L.close()
