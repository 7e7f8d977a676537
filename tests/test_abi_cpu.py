"""The C-ABI library loads, exports every declared symbol, and rejects bad arguments before touching the
device (no GPU needed; no compute call is made)."""
import ctypes as C
import os
import re

import pytest

from paper_2604_06832_amd import binding, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return binding.lib()


def _declared():
    names = set()
    for h in ("bd.h", "bd_kernels.h"):
        txt = open(os.path.join(ROOT, "include", h)).read()
        txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
        names |= set(re.findall(r"\b(bd_[a-z_0-9]+)\s*\(", txt))
    return names


def test_every_declared_symbol_is_exported_and_bound(L):
    decl = _declared()
    assert decl == set(binding.EXPORTS)
    for s in decl:
        assert hasattr(L, s), s


def test_error_strings(L):
    assert L.bd_strerror(0) == b"ok"
    for code in range(-5, 0):
        assert L.bd_strerror(code) not in (b"ok", b"unknown error")
    assert L.bd_strerror(-99) == b"unknown error"


def _cfg(**kw):
    s = inputs.TINY
    base = dict(n_layers=s.n_layers, hidden=s.hidden, n_q_heads=s.n_q_heads, n_kv_heads=s.n_kv_heads,
                head_dim=s.head_dim, ffn=s.ffn, vocab=s.vocab, rope_theta=s.rope_theta, rms_eps=s.rms_eps,
                max_seq=256, max_block=32, mask_token_id=-1, weight_dtype=binding.BD_BF16, flags=0)
    base.update(kw)
    return binding.bd_config(**base)


@pytest.mark.parametrize("bad", [dict(head_dim=48), dict(n_q_heads=3), dict(n_q_heads=2, n_kv_heads=2), dict(hidden=250), dict(max_block=0),
                                 dict(max_block=65), dict(max_seq=8), dict(vocab=1000), dict(ffn=100),
                                 dict(mask_token_id=1024), dict(n_layers=0), dict(rope_theta=0.0), dict(flags=1 << 20)])
def test_create_rejects_bad_shapes_before_any_device_call(L, bad):
    h = C.c_void_p()
    cfg = _cfg(**bad)
    assert L.bd_create(C.byref(cfg), None, C.byref(h)) == binding.BD_E_ARG
    assert not h.value


def test_create_rejects_null_and_unbuilt_dtype(L):
    h = C.c_void_p()
    assert L.bd_create(None, None, C.byref(h)) == binding.BD_E_ARG
    cfg = _cfg()
    assert L.bd_create(C.byref(cfg), None, None) == binding.BD_E_ARG
    cfg = _cfg(weight_dtype=binding.BD_F32)
    assert L.bd_create(C.byref(cfg), None, C.byref(h)) == binding.BD_E_DTYPE


def test_null_context_is_an_argument_error(L):
    assert L.bd_prefill(None, None, 0, None, 0) == binding.BD_E_ARG
    assert L.bd_denoise_step(None, None, None, 4, 0.9, 0, None, None) == binding.BD_E_ARG
    assert L.bd_commit_block(None, None, 4) == binding.BD_E_ARG
    assert L.bd_verify_block(None, None, 4, 1, None, None) == binding.BD_E_ARG
    assert L.bd_crop(None, 0) == binding.BD_E_ARG
    assert L.bd_cache_len(None) == binding.BD_E_ARG
    assert L.bd_status(None) == binding.BD_E_ARG
    assert L.bd_load_weight(None, b"embed", None, 0, 0, None) == binding.BD_E_ARG
    assert L.bd_k_attention(None, None, None, None, 0, 4, 4, 2, 64, 0, None, 1, None) == binding.BD_E_ARG
    assert L.bd_k_attention_static(None, None, None, None, 0, 4, 4, 2, 64, 0, None) == binding.BD_E_ARG
    assert L.bd_kv_page_order(None, None, 0) == binding.BD_E_ARG
    assert L.bd_k_raise_device_error(None) == binding.BD_E_ARG
    assert L.bd_kv_pages(None, None, 0) == binding.BD_E_ARG
    L.bd_destroy(None)


def test_without_a_device_create_fails_cleanly(L):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present")
    h = C.c_void_p()
    cfg = _cfg()
    assert L.bd_create(C.byref(cfg), None, C.byref(h)) == binding.BD_E_HIP
    assert L.bd_last_error()
