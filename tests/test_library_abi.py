"""CPU-side checks of the boundary: the shared library loads and exports every symbol include/wsvd.h
declares, the binding mirrors them, and host-only calls validate their arguments (no kernel is launched)."""
import ctypes
import os
import re

import pytest

import paper_2604_02570_amd as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    """Every function include/*.h declares: the product boundary (wsvd.h) and the test / profiling hooks (wsvd_test.h)."""
    names = set()
    for header in ("wsvd.h", "wsvd_test.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(wsvd_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_exported_and_bound():
    names = declared_functions()
    assert "wsvd_latent_append" in names and "wsvd_decode_attn" in names and len(names) >= 14
    lib = W.lib()
    for n in names:
        assert hasattr(lib, n), f"libwsvd.so does not export {n}"
        assert hasattr(W, n) or n == "wsvd_status_str", f"python binding lacks {n}"
    assert sorted(W.EXPORTS) == names


def test_status_strings():
    for code in range(9):
        assert W.status_str(code) != "unknown status"
    assert W.status_str(99) == "unknown status"


def test_struct_sizes_match_header():
    assert ctypes.sizeof(W.LayerDesc) == 13 * 4
    assert ctypes.sizeof(W.Cache) == 5 * ctypes.sizeof(ctypes.c_void_p)


def test_host_only_validation_and_sizes():
    d = W.layer_desc(16, 32, 32, 128, 4096, 32, 2048, "i8", "bf16", "bf16", "i8")
    codes, meta = W.wsvd_cache_bytes(d)
    assert codes == 16 * 32 * 2048 * 32 and meta == 16 * 32 * 2048 * 2
    assert 2 * (codes + meta) == 71303168          # bytes one attention call streams at this shape
    d4 = W.layer_desc(64, 32, 32, 128, 4096, 32, 4160, "i4", "bf16", "bf16", "i8")
    codes, meta = W.wsvd_cache_bytes(d4)
    assert codes == 64 * 32 * 4160 * 16 and meta == 64 * 32 * 4160 * 4
    assert W.wsvd_workspace_bytes(d) >= 65536
    for kw, status in ((dict(d_head=96), 2), (dict(rank=48), 2), (dict(n_q_heads=33), 2), (dict(t_cap=100), 2),
                       (dict(latent_dtype="i4", rank=64), 6), (dict(factor_dtype="f32"), 3), (dict(out_dtype="i8"), 3)):
        args = dict(batch=16, n_q_heads=32, n_kv_heads=32, d_head=128, d_model=4096, rank=32, t_cap=2048, latent_dtype="i8",
                    factor_dtype="bf16", x_dtype="bf16", q_dtype="i8", out_dtype="f32")
        args.update(kw)
        with pytest.raises(W.WsvdError) as e:
            W.wsvd_cache_bytes(W.layer_desc(**args))
        assert e.value.status == status, kw
    with pytest.raises(W.WsvdError) as e:
        W.wsvd_ctx_set_option(None, "max_threads", 256)        # a context is required: the setting lives in it
    assert e.value.status == W.E_NULL
