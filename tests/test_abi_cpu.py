"""No-GPU checks of the boundary: the library loads, exports every symbol the header
declares, and its host-side argument checks and arena arithmetic hold."""
import ctypes as C
import os
import re

import pytest

import paper_2505_13109_amd as fkv
from paper_2505_13109_amd.binding import FkvConfig

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_symbols():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))) if h.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fkv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = fkv.lib()
    declared = _header_symbols()
    assert declared and set(declared) == set(fkv.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(L, name) is not None


def _cfg(**kw):
    base = dict(n_layers=2, batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, page_size=32,
                max_ctx=4096, budget_tokens=512, sink_tokens=32, window_tokens=32, dtype=1,
                placement=0, tau=0.8, recall_mode=0, select_pooling=0, corr_pooling=0)
    base.update(kw)
    return FkvConfig(**base)


def test_arena_bytes_and_config_checks():
    L = fkv.lib()
    dev, host = C.c_size_t(), C.c_size_t()
    assert L.fkv_arena_bytes(C.byref(_cfg()), C.byref(dev), C.byref(host)) == 0
    # the KV store dominates: layers * heads * pages * 16 KiB per (page, KV head) unit
    store = 2 * 8 * (4096 // 32) * 16384
    assert store <= dev.value < store * 1.2 and host.value == 0
    assert L.fkv_arena_bytes(C.byref(_cfg(placement=1)), C.byref(dev), C.byref(host)) == 0
    assert host.value == store                      # whole pool on the host, 2*p*d contiguous elements per unit
    gpu_units = 32 // 32 + (32 // 32 + 2) + 2 * 14  # sink + window ring + double-buffered page cache
    assert dev.value >= 2 * 8 * gpu_units * 16384 and dev.value < store
    for bad in (dict(head_dim=64), dict(page_size=16), dict(n_q_heads=30), dict(n_q_heads=128),
                dict(max_ctx=100), dict(budget_tokens=48), dict(dtype=3), dict(placement=2),
                dict(sink_tokens=40), dict(n_layers=0), dict(recall_mode=7), dict(select_pooling=6),
                dict(select_pooling=-1), dict(corr_pooling=3), dict(placement=1, batch=4096)):
        assert L.fkv_arena_bytes(C.byref(_cfg(**bad)), C.byref(dev), C.byref(host)) == -1, bad
        assert L.fkv_last_error(None)


def test_create_rejects_bad_arenas_without_touching_the_gpu():
    L = fkv.lib()
    h = C.c_void_p()
    assert L.fkv_create(C.byref(_cfg()), None, 0, None, 0, C.byref(h)) == -1
    assert L.fkv_create(C.byref(_cfg()), C.c_void_p(0x1000100), 16, None, 0, C.byref(h)) == -4
    assert L.fkv_create(C.byref(_cfg()), C.c_void_p(0x1000101), 1 << 40, None, 0, C.byref(h)) == -1
    assert not h.value
    assert L.fkv_destroy(None) == -1 and L.fkv_context_len(None, 0) == -1


def test_binding_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(fkv.FreeKVError):
        fkv.FreeKV(n_layers=1, batch=1, n_q_heads=4, n_kv_heads=1, max_ctx=256, budget=128, sink=32,
                   window=32, tau=0.8)
