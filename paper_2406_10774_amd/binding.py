"""ctypes binding of libquest.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/quest.h and does nothing but turn torch tensors into device pointers,
pass the current HIP stream, and raise QuestError on a non-zero status.  All
computation happens in the HIP kernels; there is no fallback path: if the
library has not been built, loading fails."""
from __future__ import annotations

import ctypes
import os

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libquest.so")

QUEST_OK = 0
QUEST_FLAG_SEPARATE_LAUNCHES = 1
QUEST_FLAG_DEVICE_FENCES = 2
QUEST_FLAG_KEEP_FIRST_PAGE = 4
QUEST_FLAG_KEEP_NEWEST_PAGE = 8
STATUS_NAMES = {0: "QUEST_OK", -1: "QUEST_ERR_NULL", -2: "QUEST_ERR_SHAPE",
                -3: "QUEST_ERR_UNSUPPORTED", -4: "QUEST_ERR_WORKSPACE", -5: "QUEST_ERR_HIP"}

EXPORTS = ("quest_workspace_bytes", "quest_build_meta", "quest_append_meta", "quest_estimate",
           "quest_append_estimate", "quest_topk", "quest_topk_workspace_bytes", "quest_sparse_decode",
           "quest_select_decode", "quest_step_workspace_bytes", "quest_decode_step",
           "quest_decode_step_static", "quest_last_error")


class QuestError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class quest_cache(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("max_pages_per_seq", ctypes.c_int32), ("flags", ctypes.c_int32),
        ("num_phys_pages", ctypes.c_int64),
        ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p), ("meta", ctypes.c_void_p),
        ("page_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("num_kv_heads", ctypes.c_int32),
    ]


_lib = None


def load():
    """Load libquest.so (built by paper_2406_10774_amd.build); fail loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2406_10774_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
    cp = ctypes.POINTER(quest_cache)
    lib.quest_workspace_bytes.argtypes = [cp, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.quest_build_meta.argtypes = [cp, vp]
    lib.quest_append_meta.argtypes = [cp, vp, vp, i32, vp]
    lib.quest_estimate.argtypes = [cp, vp, vp, vp]
    lib.quest_append_estimate.argtypes = [cp, vp, vp, i32, vp, vp, vp]
    lib.quest_topk.argtypes = [cp, vp, i32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.quest_topk_workspace_bytes.argtypes = [cp, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.quest_sparse_decode.argtypes = [cp, vp, vp, i32, f32, vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.quest_select_decode.argtypes = [cp, vp, vp, i32, f32, vp, vp, vp, i32, vp, vp, ctypes.c_size_t, vp]
    lib.quest_step_workspace_bytes.argtypes = [cp, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.quest_decode_step.argtypes = [cp, vp, vp, i32, vp, i32, f32, vp, vp, vp, vp, i32, vp, vp,
                                      ctypes.c_size_t, vp]
    lib.quest_decode_step_static.argtypes = [cp, vp, vp, i32, vp, i32, f32, vp, vp, vp, vp, i32, vp, vp]
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ctypes.c_int
    lib.quest_last_error.argtypes = []
    lib.quest_last_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(int(stream))
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status):
    if status != QUEST_OK:
        raise QuestError(status, load().quest_last_error().decode())


class Cache:
    """Host-side description of one layer's paged KV cache (see quest_cache in quest.h).

    Holds references to the caller's torch tensors so they outlive the calls."""

    def __init__(self, k_pool, v_pool, meta, page_table, seq_lens, flags=0, num_heads=None):
        """num_heads: query heads, if more than the KV heads of the pools (grouped-query
        attention); default: one KV head per query head."""
        N, Hkv, S, D = k_pool.shape
        H = Hkv if num_heads is None else int(num_heads)
        self.k_pool, self.v_pool, self.meta = k_pool, v_pool, meta
        self.page_table, self.seq_lens = page_table, seq_lens
        self.c = quest_cache(
            batch=page_table.shape[0], num_heads=H, head_dim=D, page_size=S,
            max_pages_per_seq=page_table.shape[1], flags=int(flags), num_phys_pages=N,
            k_pool=k_pool.data_ptr(), v_pool=v_pool.data_ptr() if v_pool is not None else None,
            meta=meta.data_ptr(), page_table=page_table.data_ptr(), seq_lens=seq_lens.data_ptr(),
            num_kv_heads=0 if H == Hkv else Hkv)

    @property
    def ref(self):
        return ctypes.byref(self.c)


def quest_workspace_bytes(cache: Cache, k_pages: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().quest_workspace_bytes(cache.ref, int(k_pages), ctypes.byref(out)))
    return out.value


def quest_build_meta(cache: Cache, stream=None):
    _check(load().quest_build_meta(cache.ref, _stream(stream)))


def quest_append_meta(cache: Cache, k_new, v_new=None, k_pool_write=False, stream=None):
    _check(load().quest_append_meta(cache.ref, _ptr(k_new), _ptr(v_new), int(bool(k_pool_write)),
                                    _stream(stream)))


def quest_estimate(cache: Cache, q, scores, stream=None):
    _check(load().quest_estimate(cache.ref, _ptr(q), _ptr(scores), _stream(stream)))


def quest_append_estimate(cache: Cache, k_new, v_new, k_pool_write, q, scores, stream=None):
    _check(load().quest_append_estimate(cache.ref, _ptr(k_new), _ptr(v_new),
                                        int(bool(k_pool_write)), _ptr(q), _ptr(scores),
                                        _stream(stream)))


def quest_topk(cache: Cache, scores, k_pages, topk_idx, k_eff=None, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().quest_topk(cache.ref, _ptr(scores), int(k_pages), _ptr(topk_idx), _ptr(k_eff),
                             _ptr(workspace), ws_bytes, _stream(stream)))


def quest_topk_workspace_bytes(cache: Cache, k_pages: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().quest_topk_workspace_bytes(cache.ref, int(k_pages), ctypes.byref(out)))
    return out.value


def quest_sparse_decode(cache: Cache, q, topk_idx, k_pages, sm_scale, out, lse=None,
                        workspace=None, stream=None):
    import torch
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().quest_sparse_decode(
        cache.ref, _ptr(q), _ptr(topk_idx), int(k_pages), float(sm_scale), _ptr(out),
        int(out.dtype == torch.float16), _ptr(lse), _ptr(workspace), ws_bytes, _stream(stream)))


def quest_select_decode(cache: Cache, q, scores, k_pages, sm_scale, topk_idx, out, k_eff=None,
                        lse=None, workspace=None, stream=None):
    import torch
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().quest_select_decode(
        cache.ref, _ptr(q), _ptr(scores), int(k_pages), float(sm_scale), _ptr(topk_idx), _ptr(k_eff),
        _ptr(out), int(out.dtype == torch.float16), _ptr(lse), _ptr(workspace), ws_bytes,
        _stream(stream)))


def quest_step_workspace_bytes(cache: Cache, k_pages: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().quest_step_workspace_bytes(cache.ref, int(k_pages), ctypes.byref(out)))
    return out.value


def quest_decode_step(cache: Cache, k_new, v_new, k_pool_write, q, k_pages, sm_scale, scores,
                      topk_idx, out, workspace, k_eff=None, lse=None, stream=None):
    import torch
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(load().quest_decode_step(
        cache.ref, _ptr(k_new), _ptr(v_new), int(bool(k_pool_write)), _ptr(q), int(k_pages),
        float(sm_scale), _ptr(scores), _ptr(topk_idx), _ptr(k_eff), _ptr(out),
        int(out.dtype == torch.float16), _ptr(lse), _ptr(workspace), ws_bytes, _stream(stream)))



def quest_decode_step_static(cache: Cache, k_new, v_new, k_pool_write, q, k_pages, sm_scale, scores,
                             topk_idx, out, k_eff=None, lse=None, stream=None):
    import torch
    _check(load().quest_decode_step_static(
        cache.ref, _ptr(k_new), _ptr(v_new), int(bool(k_pool_write)), _ptr(q), int(k_pages),
        float(sm_scale), _ptr(scores), _ptr(topk_idx), _ptr(k_eff), _ptr(out),
        int(out.dtype == torch.float16), _ptr(lse), _stream(stream)))
