"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared
symbol, and rejects bad arguments with the documented codes before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2501_08090_amd import binding as B
from paper_2501_08090_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for h in ("chiron.h", "chiron_ops.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(chiron_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    lib = B.load()
    decl = declared_symbols()
    assert decl == set(B.SYMBOLS), "binding.SYMBOLS and the headers disagree: %s" % (decl ^ set(B.SYMBOLS))
    for s in decl:
        assert hasattr(lib, s), s


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libchiron.so")
    with pytest.raises(ImportError):
        B.load()


def test_bad_configs_are_rejected_without_a_device():
    lib = B.load()
    h = C.c_void_p()
    ok = dict(I.TINY)
    cases = [
        (dict(ok, head_dim=96), -2), (dict(ok, n_q_heads=3), -2), (dict(ok, n_q_heads=6, n_kv_heads=2), -2),
        (dict(ok, hidden=250), -2), (dict(ok, ffn=690), -2), (dict(ok, n_layers=0), -1), (dict(ok, rope_base=1.0), -1),
    ]
    for m, code in cases:
        cfg = B.make_config(m, 4, 8)
        assert lib.chiron_model_create(C.byref(cfg), C.byref(h)) == code, m
        assert h.value is None and B.last_error() != ""
    cfg = B.make_config(ok, 4, 8)
    cfg.dtype = 7
    assert lib.chiron_model_create(C.byref(cfg), C.byref(h)) == -1
    assert lib.chiron_model_create(None, C.byref(h)) == -1
    assert lib.chiron_model_create(C.byref(cfg), None) == -1


def test_null_handles_are_invalid_arguments():
    lib = B.load()
    z = C.c_void_p(0)
    assert lib.chiron_decode_step(z, z, z, z, z, C.c_int32(1), z, z) == -1
    assert lib.chiron_append_kv(z, 0, z, z, z, 1, z, z, C.c_int64(1), z) == -1
    assert lib.chiron_gather_kv(z, 0, z, 1, z, z, z) == -1
    assert lib.chiron_kv_pool_create(z, z, C.c_uint64(0), 16, C.byref(C.c_void_p()), None) == -1
    assert lib.chiron_op_linear(z, z, 1, z, 0, z) == -1
    assert lib.chiron_set_tuning(b"no_such_knob", 1) == -1
    assert lib.chiron_set_tuning(None, 1) == -1
    # a knob takes only the values a kernel shape exists for; a rejected value leaves the knob as it was
    for key, bad in ((b"linear_nf", 3), (b"linear_nf", 8), (b"linear_mt", 5), (b"linear_mt", -1), (b"linear_ks", 6),
                     (b"linear_ksplit", 17), (b"attn_grid", -1), (b"linear_xcd_remap", 2), (b"attn_chunk_pages", -2)):
        assert lib.chiron_set_tuning(key, bad) == -1 and b"not allowed" in lib.chiron_last_error()
    for key, ok in ((b"linear_nf", 4), (b"linear_mt", 3), (b"linear_ks", 8), (b"linear_ks", 16), (b"linear_big_min_m", -1), (b"attn_grid", 7)):
        assert lib.chiron_set_tuning(key, ok) == 0
        assert lib.chiron_set_tuning(key, 0) == 0
    assert lib.chiron_model_destroy(z) == 0 and lib.chiron_kv_pool_destroy(z) == 0 and lib.chiron_linear_destroy(z) == 0


def test_host_validation_of_index_arrays():
    cfg = B.make_config(I.TINY, 4, 4)
    lens = np.array([5, 16, 40], np.int32)
    bt = np.array([[3, -1, -1, -1], [0, 1, -1, -1], [2, 4, 5, -1]], np.int32)
    tok = np.array([1, 2, 3], np.int32)
    chk = lambda **k: B.check_step_inputs_host(cfg, k.get("nb", 6), k.get("bt", bt), k.get("lens", lens), k.get("tok", tok))
    assert chk() == 0
    assert chk(tok=np.array([1, 1024, 3], np.int32)) == -7 and "tokens[1]" in B.last_error()
    assert chk(tok=np.array([-1, 2, 3], np.int32)) == -7
    assert chk(nb=5) == -4                                        # page 5 is not in a 5-page pool
    b2 = bt.copy(); b2[1, 1] = -1
    assert chk(bt=b2) == -4                                       # position 16 needs a second page
    assert chk(lens=np.array([5, 16, 70], np.int32)) == -4        # 71 tokens need 5 pages, rows hold 4
    b3 = bt.copy(); b3[0, 0] = 1
    assert chk(bt=b3) == -4 and "more than one" in B.last_error() # two requests write page 1
    b4 = bt.copy(); b4[2, 0] = 3
    assert chk(bt=b4) == -4                                       # request 2 reads the page request 0 writes
    shared = np.array([[0, 1, -1, -1], [0, 2, -1, -1]], np.int32)  # read-only shared first page is fine
    assert B.check_step_inputs_host(cfg, 3, shared, np.array([20, 17], np.int32), np.array([0, 0], np.int32)) == 0
    assert chk(lens=np.array([5, -1, 40], np.int32)) == -1
    big = np.zeros(5, np.int32)
    assert B.check_step_inputs_host(cfg, 6, np.zeros((5, 4), np.int32), big, big) == -3


def test_host_validation_of_multi_token_inputs():
    """positions L .. L+q_len-1 are written: their pages must exist and belong to one request only"""
    cfg = B.make_config(I.TINY, 12, 4)
    lens = np.array([5, 14, 40], np.int32)
    bt = np.array([[3, -1, -1, -1], [0, 1, -1, -1], [2, 4, 5, -1]], np.int32)
    tok = np.arange(9, dtype=np.int32).reshape(3, 3)
    chk = lambda **k: B.check_step_inputs_host(cfg, k.get("nb", 6), k.get("bt", bt), k.get("lens", lens), k.get("tok", tok))
    assert chk() == 0                                             # request 1 writes positions 14, 15, 16: pages 0 and 1
    b2 = bt.copy(); b2[1, 1] = -1
    assert chk(bt=b2) == -4                                       # ... so its second page must exist
    assert B.check_step_inputs_host(cfg, 6, b2, lens, tok[:, :2]) == 0   # two tokens stay in the first page
    b3 = bt.copy(); b3[0, 0] = 1
    assert chk(bt=b3) == -4 and "more than one" in B.last_error() # page 1 is written by requests 0 and 1
    t2 = tok.copy(); t2[2, 2] = 5000
    assert chk(tok=t2) == -7 and "tokens[8]" in B.last_error()
    assert chk(lens=np.array([5, 14, 62], np.int32)) == -4        # 62 + 3 positions need 5 pages, rows hold 4
    assert B.check_step_inputs_host(cfg, 6, np.zeros((5, 4), np.int32), np.zeros(5, np.int32), np.zeros((5, 3), np.int32)) == -3

