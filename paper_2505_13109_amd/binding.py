"""ctypes binding of include/freekv.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# PyTorch supplies device memory and streams, so the library must share its HIP runtime:
# torch is imported first and libfreekv.so then binds to the libamdhip64 already loaded.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))

FKV_DTYPE_FP16, FKV_DTYPE_BF16 = 0, 1
FKV_PLACE_HBM, FKV_PLACE_HOST = 0, 1
FKV_USE_ACTIVE, FKV_USE_PENDING, FKV_USE_BY_FLAG = 0, 1, 2
FKV_HEADS_ALL, FKV_HEADS_FLAGGED, FKV_HEADS_UNFLAGGED = 0, 1, 2
FKV_RECALL_GATHER, FKV_RECALL_MEMCPY = 0, 1
DBG_SUMMARIES, DBG_WEIGHTS, DBG_SCORES, DBG_ACTIVE_IDS, DBG_PENDING_IDS, DBG_FLAGS, DBG_MISS, DBG_COSINE, DBG_TSTAMP = range(9)

EXPORTED_SYMBOLS = (
    "fkv_arena_bytes", "fkv_create", "fkv_destroy", "fkv_last_error", "fkv_context_len", "fkv_health",
    "fkv_load_prefix", "fkv_kv_append", "fkv_page_summary_update", "fkv_corr_check",
    "fkv_page_select", "fkv_recall_pages", "fkv_sparse_decode_attn", "fkv_commit",
    "fkv_decode_step", "fkv_flush", "fkv_debug_read", "fkv_debug_read_page", "fkv_profile_enable", "fkv_profile_read", "fkv_profile_attn", "fkv_profile_select", "fkv_profile_launch_floor", "fkv_step_launches", "fkv_export_nhd",
    "fkv_sparse_decode_attn_static", "fkv_recall_pending", "fkv_attach_nhd_pool", "fkv_test_lose_selection", "fkv_instrument_timestamps",
)


class FreeKVError(RuntimeError):
    pass


# names of the FKV_POOL_* / FKV_CORR_* codes, in code order
SELECT_POOLINGS = ("MeanS", "MaxS", "MeanQK", "MaxQK", "MeanQ", "MaxQ")
CORR_POOLINGS = ("mean", "max", "min")


class FkvConfig(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("page_size", C.c_int32),
        ("max_ctx", C.c_int32), ("budget_tokens", C.c_int32), ("sink_tokens", C.c_int32),
        ("window_tokens", C.c_int32), ("dtype", C.c_int32), ("placement", C.c_int32),
        ("tau", C.c_float), ("recall_mode", C.c_int32), ("select_pooling", C.c_int32), ("corr_pooling", C.c_int32),
    ]


def lib_path() -> str:
    """The in-tree library; FKV_LIB names another build of it (experiments)."""
    return os.environ.get("FKV_LIB") or os.path.join(_HERE, "libfreekv.so")


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FreeKVError(f"{path} is missing: build it with `python -m paper_2505_13109_amd.build`")
    L = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    cfgp = C.POINTER(FkvConfig)
    sig = {
        "fkv_arena_bytes": (C.c_int, [cfgp, C.POINTER(sz), C.POINTER(sz)]),
        "fkv_create": (C.c_int, [cfgp, vp, sz, vp, sz, C.POINTER(vp)]),
        "fkv_destroy": (C.c_int, [vp]),
        "fkv_last_error": (C.c_char_p, [vp]),
        "fkv_context_len": (C.c_int, [vp, i32]),
        "fkv_health": (C.c_int, [vp, i32]),
        "fkv_step_launches": (C.c_int, [vp, i32]),
        "fkv_flush": (C.c_int, [vp]),
        "fkv_load_prefix": (C.c_int, [vp, i32, vp, vp, i32, vp]),
        "fkv_kv_append": (C.c_int, [vp, i32, vp, vp, vp, vp]),
        "fkv_page_summary_update": (C.c_int, [vp, i32, i32, i32, vp]),
        "fkv_corr_check": (C.c_int, [vp, i32, vp, vp, vp]),
        "fkv_page_select": (C.c_int, [vp, i32, vp, vp, vp]),
        "fkv_recall_pages": (C.c_int, [vp, i32, vp, vp, vp]),
        "fkv_recall_pending": (C.c_int, [vp, i32, i32, vp]),
        "fkv_attach_nhd_pool": (C.c_int, [vp, vp, vp, i32]),
        "fkv_test_lose_selection": (C.c_int, [vp, i32]),
        "fkv_instrument_timestamps": (C.c_int, [vp, i32]),
        "fkv_sparse_decode_attn": (C.c_int, [vp, i32, vp, vp, i32, vp]),
        "fkv_sparse_decode_attn_static": (C.c_int, [vp, i32, vp, vp, i32, vp]),
        "fkv_commit": (C.c_int, [vp, i32]),
        "fkv_decode_step": (C.c_int, [vp, i32, vp, vp, vp, vp, vp, vp]),
        "fkv_export_nhd": (C.c_int, [vp, i32, i32, vp, vp, i32, vp]),
        "fkv_profile_enable": (C.c_int, [vp, i32]),
        "fkv_profile_read": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(i32)]),
        "fkv_profile_attn": (C.c_int, [vp, vp, sz, vp, i32, vp, C.POINTER(C.c_double), C.POINTER(i32)]),
        "fkv_profile_select": (C.c_int, [vp, vp, sz, i32, vp, C.POINTER(C.c_double), C.POINTER(i32)]),
        "fkv_profile_launch_floor": (C.c_int, [vp, i32, i32, vp, C.POINTER(C.c_double), C.POINTER(i32), C.POINTER(i32)]),
        "fkv_debug_read": (C.c_int, [vp, i32, i32, vp, sz]),
        "fkv_debug_read_page": (C.c_int, [vp, i32, i32, i32, i32, i32, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(s):
    if s is None:
        import torch
        s = torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


class FreeKV:
    """One context.  Methods carry the names of the C entry points they call."""

    def __init__(self, *, n_layers, batch, n_q_heads, n_kv_heads, max_ctx, budget, sink, window,
                 tau, dtype="bf16", placement=FKV_PLACE_HBM, head_dim=128, page_size=32, device="cuda:0",
                 recall_mode=0, select_pooling="MeanS", corr_pooling="mean"):
        import torch
        self._torch = torch
        self.L = lib()
        self.cfg = FkvConfig(n_layers, batch, n_q_heads, n_kv_heads, head_dim, page_size, max_ctx,
                             budget, sink, window, {"fp16": 0, "bf16": 1}[dtype], placement, tau, recall_mode,
                             SELECT_POOLINGS.index(select_pooling), CORR_POOLINGS.index(corr_pooling))
        self.dtype = dtype
        self.torch_dtype = torch.float16 if dtype == "fp16" else torch.bfloat16
        self.k = (budget - sink - window) // page_size
        self.max_pages = max_ctx // page_size
        self.device = torch.device(device)
        self._h = C.c_void_p()
        dev_b, host_b = C.c_size_t(), C.c_size_t()
        rc = self.L.fkv_arena_bytes(C.byref(self.cfg), C.byref(dev_b), C.byref(host_b))
        if rc:
            raise FreeKVError(f"fkv_arena_bytes: {rc}: {self.L.fkv_last_error(None).decode()}")
        self.dev_bytes, self.host_bytes = dev_b.value, host_b.value
        if not torch.cuda.is_available():
            raise FreeKVError("no GPU: the FreeKV path runs only in its HIP kernels")
        torch.cuda.set_device(self.device)
        self.dev_arena = torch.empty(self.dev_bytes, dtype=torch.uint8, device=self.device)
        self.host_arena = None
        if self.host_bytes:
            self.host_arena = torch.empty(self.host_bytes, dtype=torch.uint8, pin_memory=True)
        rc = self.L.fkv_create(C.byref(self.cfg), _ptr(self.dev_arena), self.dev_bytes,
                               _ptr(self.host_arena), self.host_bytes, C.byref(self._h))
        if rc:
            raise FreeKVError(f"fkv_create: {rc}: {self.L.fkv_last_error(None).decode()}")

    # -- plumbing ------------------------------------------------------------
    def _check(self, rc, what):
        if rc:
            raise FreeKVError(f"{what}: {rc}: {self.L.fkv_last_error(self._h).decode()}")

    def close(self):
        if self._h:
            self.L.fkv_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- entry points ---------------------------------------------------------
    def context_len(self, layer):
        return self.L.fkv_context_len(self._h, layer)

    def step_launches(self, layer):
        return self.L.fkv_step_launches(self._h, layer)

    def load_prefix(self, layer, K, V, stream=None):
        assert K.is_contiguous() and V.is_contiguous() and K.dtype == self.torch_dtype
        self._check(self.L.fkv_load_prefix(self._h, layer, _ptr(K), _ptr(V), K.shape[1], _stream(stream)), "fkv_load_prefix")

    def kv_append(self, layer, k_new, v_new, stream=None, copy_stream=None):
        s = _stream(stream)
        cs = s if copy_stream is None else _stream(copy_stream)
        self._check(self.L.fkv_kv_append(self._h, layer, _ptr(k_new), _ptr(v_new), s, cs), "fkv_kv_append")

    def page_summary_update(self, layer, first_page, n_pages, stream=None):
        self._check(self.L.fkv_page_summary_update(self._h, layer, first_page, n_pages, _stream(stream)), "fkv_page_summary_update")

    def corr_check(self, layer, q, flags=None, stream=None):
        self._check(self.L.fkv_corr_check(self._h, layer, _ptr(q), _ptr(flags), _stream(stream)), "fkv_corr_check")

    def page_select(self, layer, q, page_ids=None, stream=None):
        self._check(self.L.fkv_page_select(self._h, layer, _ptr(q), _ptr(page_ids), _stream(stream)), "fkv_page_select")

    def recall_pages(self, layer, page_ids=None, head_mask=None, copy_stream=None):
        self._check(self.L.fkv_recall_pages(self._h, layer, _ptr(page_ids), _ptr(head_mask), _stream(copy_stream)), "fkv_recall_pages")

    def recall_pending(self, layer, heads=FKV_HEADS_ALL, copy_stream=None):
        self._check(self.L.fkv_recall_pending(self._h, layer, heads, _stream(copy_stream)), "fkv_recall_pending")

    def test_lose_selection(self, on):
        self._check(self.L.fkv_test_lose_selection(self._h, int(on)), "fkv_test_lose_selection")

    def instrument_timestamps(self, on):
        self._check(self.L.fkv_instrument_timestamps(self._h, int(on)), "fkv_instrument_timestamps")

    def sparse_decode_attn(self, layer, q, out, use=FKV_USE_ACTIVE, stream=None):
        self._check(self.L.fkv_sparse_decode_attn(self._h, layer, _ptr(q), _ptr(out), use, _stream(stream)), "fkv_sparse_decode_attn")

    def sparse_decode_attn_static(self, layer, q, out, use=FKV_USE_ACTIVE, stream=None):
        self._check(self.L.fkv_sparse_decode_attn_static(self._h, layer, _ptr(q), _ptr(out), use, _stream(stream)),
                    "fkv_sparse_decode_attn_static")

    def export_nhd(self, layer, nhd_pool, slot_pages, use=FKV_USE_ACTIVE, stream=None):
        """nhd_pool [batch, n_slots, 2, page, n_kv, d] storage type, slot_pages [batch, n_kv, n_slots] int32."""
        self._check(self.L.fkv_export_nhd(self._h, layer, use, _ptr(nhd_pool), _ptr(slot_pages),
                                          slot_pages.shape[-1], _stream(stream)), "fkv_export_nhd")

    def attach_nhd_pool(self, nhd_pool, slot_pages):
        """Streamed recall into this NHD pool from now on (None, None detaches); shapes as in export_nhd."""
        n_slots = 0 if slot_pages is None else slot_pages.shape[-1]
        self._nhd_keep = (nhd_pool, slot_pages)          # the library only keeps the addresses
        self._check(self.L.fkv_attach_nhd_pool(self._h, _ptr(nhd_pool), _ptr(slot_pages), n_slots), "fkv_attach_nhd_pool")

    def commit(self, layer):
        self._check(self.L.fkv_commit(self._h, layer), "fkv_commit")

    def decode_step(self, layer, q, k_new, v_new, out, stream=None, copy_stream=None):
        s = _stream(stream)
        cs = s if copy_stream is None else _stream(copy_stream)
        self._check(self.L.fkv_decode_step(self._h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), s, cs), "fkv_decode_step")

    def flush(self):
        self._check(self.L.fkv_flush(self._h), "fkv_flush")

    def profile_enable(self, max_launches):
        self._check(self.L.fkv_profile_enable(self._h, max_launches), "fkv_profile_enable")

    def profile_read(self):
        ms, n = C.c_double(), C.c_int32()
        self._check(self.L.fkv_profile_read(self._h, C.byref(ms), C.byref(n)), "fkv_profile_read")
        return ms.value, n.value

    def profile_launch_floor(self, layer, reps, stream=None):
        """(ms for `reps` empty launches of the layer kernel's shape, grid, dynamic LDS bytes)"""
        ms, grid, lds = C.c_double(), C.c_int32(), C.c_int32()
        self._check(self.L.fkv_profile_launch_floor(self._h, layer, reps, _stream(stream), C.byref(ms),
                                                    C.byref(grid), C.byref(lds)), "fkv_profile_launch_floor")
        return ms.value, grid.value, lds.value

    def profile_attn(self, q_layers, out, reps, stream=None):
        """q_layers: [n_layers, batch, n_q, d] contiguous; returns (total_ms, launches)."""
        ms, n = C.c_double(), C.c_int32()
        stride = q_layers.stride(0) * q_layers.element_size()
        self._check(self.L.fkv_profile_attn(self._h, _ptr(q_layers), stride, _ptr(out), reps, _stream(stream),
                                            C.byref(ms), C.byref(n)), "fkv_profile_attn")
        return ms.value, n.value

    def profile_select(self, q_layers, reps, stream=None):
        """q_layers: [n_layers, batch, n_q, d] contiguous; returns (total_ms, launches) of scan + selection."""
        ms, n = C.c_double(), C.c_int32()
        stride = q_layers.stride(0) * q_layers.element_size()
        self._check(self.L.fkv_profile_select(self._h, _ptr(q_layers), stride, reps, _stream(stream),
                                              C.byref(ms), C.byref(n)), "fkv_profile_select")
        return ms.value, n.value

    def health(self, layer):
        """Raises if a kernel of this layer gave up a bounded wait (blocking)."""
        self._check(self.L.fkv_health(self._h, layer), "fkv_health")

    # -- introspection ----------------------------------------------------------
    def debug_read(self, layer, what):
        c = self.cfg
        shapes = {
            DBG_SUMMARIES: ((c.batch, c.n_kv_heads, 2, self.max_pages, c.head_dim), np.uint16),
            DBG_WEIGHTS: ((c.batch, c.n_q_heads, self.max_pages), np.float32),
            DBG_SCORES: ((c.batch, c.n_kv_heads, self.max_pages), np.float32),
            DBG_ACTIVE_IDS: ((c.batch, c.n_kv_heads, self.k), np.int32),
            DBG_PENDING_IDS: ((c.batch, c.n_kv_heads, self.k), np.int32),
            DBG_FLAGS: ((c.batch, c.n_kv_heads), np.uint8),
            DBG_MISS: ((c.batch, c.n_kv_heads, 1 + self.k), np.int32),
            DBG_COSINE: ((c.batch, c.n_q_heads), np.float64),
            DBG_TSTAMP: ((64,), np.int64),
        }
        shape, dt = shapes[what]
        out = np.empty(shape, dtype=dt)
        self._check(self.L.fkv_debug_read(self._h, layer, what, out.ctypes.data_as(C.c_void_p), out.nbytes), "fkv_debug_read")
        return out

    def debug_read_page(self, layer, request, kv_head, page, where):
        out = np.empty((2, self.cfg.page_size, self.cfg.head_dim), dtype=np.uint16)
        self._check(self.L.fkv_debug_read_page(self._h, layer, request, kv_head, page, where, out.ctypes.data_as(C.c_void_p)), "fkv_debug_read_page")
        return out
