"""ctypes binding of libxkv.so: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxkv.so")

XKV_F32, XKV_BF16 = 0, 1
XKV_ALLOC_TOTAL_SIZE, XKV_ALLOC_TARGET_RAVG = 0, 1

EXPORTS = (
    "xkv_status_string", "xkv_allocate_budgets", "xkv_workspace_bytes",
    "xkv_decode_attend_score", "xkv_evict_compact", "xkv_profile_enable", "xkv_profile_read",
    "xkv_configure", "xkv_probe_stream_read", "xkv_prefill_workspace_bytes", "xkv_prefill_evict",
    "xkv_window_importance", "xkv_allocate_device_workspace_bytes", "xkv_allocate_budgets_device",
    "xkv_average_allocations", "xkv_fused_status", "xkv_decode_attend_score_noalloc", "xkv_repack", "xkv_cache_importance",
    "xkv_prefill_evict_lse", "xkv_window_importance_lse", "xkv_decode_step",
)
XKV_NOALLOC_SCRATCH_BYTES = 32 << 20
XKV_CFG_ATTEND_PATH = 1
XKV_CFG_FUSED_SPIN_LIMIT = 2


class XkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _CacheStruct(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("dtype", C.c_int32),
        ("arena_slots", C.c_int64),
        ("k", C.c_void_p), ("v", C.c_void_p), ("score", C.c_void_p), ("pos", C.c_void_p),
        ("region_off", C.c_void_p), ("cap", C.c_void_p), ("len", C.c_void_p),
    ]


_lib = None


def load():
    """Loads libxkv.so (built in-tree by __graft_entry__.build()).  There is no
    fallback: without the library nothing here works."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` (build()) first")
    try:
        import torch  # noqa: F401  (its HIP runtime must be the one the library binds to)
    except Exception:
        pass
    lib = C.CDLL(LIB_PATH)
    lib.xkv_status_string.restype = C.c_char_p
    lib.xkv_status_string.argtypes = [C.c_int32]
    lib.xkv_allocate_budgets.restype = C.c_int32
    lib.xkv_allocate_budgets.argtypes = [
        C.c_int32, C.POINTER(C.c_void_p), C.c_void_p, C.c_int32, C.c_int64, C.c_double,
        C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
    lib.xkv_workspace_bytes.restype = C.c_int32
    lib.xkv_workspace_bytes.argtypes = [C.POINTER(_CacheStruct), C.c_int32, C.POINTER(C.c_size_t)]
    lib.xkv_decode_attend_score.restype = C.c_int32
    lib.xkv_decode_attend_score.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
        C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xkv_decode_attend_score_noalloc.restype = C.c_int32
    lib.xkv_decode_attend_score_noalloc.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
        C.c_void_p, C.c_float, C.c_void_p, C.c_void_p]
    lib.xkv_cache_importance.restype = C.c_int32
    lib.xkv_cache_importance.argtypes = [C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                         C.c_void_p]
    lib.xkv_repack.restype = C.c_int32
    lib.xkv_repack.argtypes = [C.POINTER(_CacheStruct), C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p]
    lib.xkv_decode_step.restype = C.c_int32
    lib.xkv_decode_step.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float,
        C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xkv_evict_compact.restype = C.c_int32
    lib.xkv_evict_compact.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xkv_prefill_workspace_bytes.restype = C.c_int32
    lib.xkv_prefill_workspace_bytes.argtypes = [C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_int32,
                                                C.POINTER(C.c_size_t)]
    lib.xkv_prefill_evict.restype = C.c_int32
    lib.xkv_prefill_evict.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
        C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
        C.c_void_p]
    lib.xkv_prefill_evict_lse.restype = C.c_int32
    lib.xkv_prefill_evict_lse.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
        C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
        C.c_void_p]
    lib.xkv_window_importance_lse.restype = C.c_int32
    lib.xkv_window_importance_lse.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
        C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xkv_window_importance.restype = C.c_int32
    lib.xkv_window_importance.argtypes = [
        C.POINTER(_CacheStruct), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
        C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xkv_allocate_device_workspace_bytes.restype = C.c_int32
    lib.xkv_allocate_device_workspace_bytes.argtypes = [C.c_int32, C.c_int64, C.POINTER(C.c_size_t)]
    lib.xkv_allocate_budgets_device.restype = C.c_int32
    lib.xkv_allocate_budgets_device.argtypes = [
        C.c_int32, C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int64, C.c_double, C.c_void_p, C.c_void_p,
        C.c_void_p, C.POINTER(C.c_double), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.xkv_average_allocations.restype = C.c_int32
    lib.xkv_average_allocations.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                            C.c_void_p]
    lib.xkv_configure.restype = C.c_int32
    lib.xkv_configure.argtypes = [C.c_int32, C.c_int64]
    lib.xkv_fused_status.restype = C.c_int32
    lib.xkv_fused_status.argtypes = [C.POINTER(C.c_int32)]
    lib.xkv_probe_stream_read.restype = C.c_int32
    lib.xkv_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_void_p]
    lib.xkv_profile_enable.restype = C.c_int32
    lib.xkv_profile_enable.argtypes = [C.c_int32]
    lib.xkv_profile_read.restype = C.c_int32
    lib.xkv_profile_read.argtypes = [C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().xkv_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise XkvError(status, where)


def _ptr(t) -> Optional[int]:
    """Address of a torch tensor / numpy array (None stays NULL)."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ---------------------------------------------------------------------------
def xkv_allocate_budgets(w: Sequence[np.ndarray], mode: int = XKV_ALLOC_TOTAL_SIZE,
                         total_size: int = 0, target_ravg: float = 0.0,
                         min_budget=None, max_budget=None):
    """-> (budgets int64 [L], R_avg).  w: one fp32 vector per layer."""
    lib = load()
    L = len(w)
    arrs = [np.ascontiguousarray(x, dtype=np.float32) for x in w]
    ptrs = (C.c_void_p * max(L, 1))(*[a.ctypes.data for a in arrs])
    lens = np.asarray([a.size for a in arrs], dtype=np.int64)
    lo = None if min_budget is None else np.ascontiguousarray(min_budget, dtype=np.int64)
    hi = None if max_budget is None else np.ascontiguousarray(max_budget, dtype=np.int64)
    out = np.zeros(max(L, 1), dtype=np.int64)
    ravg = C.c_double(0.0)
    st = lib.xkv_allocate_budgets(L, ptrs, lens.ctypes.data, int(mode), int(total_size),
                                  float(target_ravg), _ptr(lo), _ptr(hi), out.ctypes.data,
                                  C.byref(ravg))
    _check(st, "xkv_allocate_budgets")
    return out[:L], ravg.value


def xkv_average_allocations(lists, total_size: int, min_budget=None, max_budget=None):
    """lists: integers [n_samples, L] -> budgets int64 [L] summing to total_size."""
    arr = np.ascontiguousarray(lists, dtype=np.int64)
    if arr.ndim != 2:
        raise ValueError("lists must be [n_samples, L]")
    lo = None if min_budget is None else np.ascontiguousarray(min_budget, dtype=np.int64)
    hi = None if max_budget is None else np.ascontiguousarray(max_budget, dtype=np.int64)
    out = np.zeros(max(arr.shape[1], 1), dtype=np.int64)
    st = load().xkv_average_allocations(arr.shape[0], arr.shape[1], arr.ctypes.data, int(total_size), _ptr(lo),
                                        _ptr(hi), out.ctypes.data)
    _check(st, "xkv_average_allocations")
    return out[:arr.shape[1]]


class XkvCache:
    """Owns the arenas (torch tensors) and the host tables of one ragged cache
    and the xkv_cache struct that points at them."""

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, dtype, caps, device="cuda", zero=True):
        """zero=False leaves the arenas uninitialised (the library never reads a slot at or beyond len)."""
        import torch
        caps = np.ascontiguousarray(caps, dtype=np.int32).reshape(n_layers * batch)
        self.n_layers, self.batch = int(n_layers), int(batch)
        self.n_q_heads, self.n_kv_heads, self.head_dim = int(n_q_heads), int(n_kv_heads), int(head_dim)
        self.dtype = dtype
        self.torch_dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
        sizes = caps.astype(np.int64) * n_kv_heads
        self.region_off = np.zeros(n_layers * batch, dtype=np.int64)
        if sizes.size > 1:
            self.region_off[1:] = np.cumsum(sizes)[:-1]
        self.cap = caps
        self.len = np.zeros(n_layers * batch, dtype=np.int32)
        self.arena_slots = int(sizes.sum())
        slots = max(self.arena_slots, 1)
        alloc = torch.zeros if zero else torch.empty
        self.k = alloc((slots, head_dim), dtype=self.torch_dtype, device=device)
        self.v = alloc((slots, head_dim), dtype=self.torch_dtype, device=device)
        self.score = alloc(slots, dtype=torch.float32, device=device)
        self.pos = alloc(slots, dtype=torch.int32, device=device)
        self.struct = _CacheStruct()
        self.refresh()

    def refresh(self):
        s = self.struct
        s.n_layers, s.batch, s.n_q_heads = self.n_layers, self.batch, self.n_q_heads
        s.n_kv_heads, s.head_dim = self.n_kv_heads, self.head_dim
        s.dtype = XKV_F32 if self.dtype == "f32" else XKV_BF16
        s.arena_slots = self.arena_slots
        s.k, s.v, s.score, s.pos = (self.k.data_ptr(), self.v.data_ptr(),
                                    self.score.data_ptr(), self.pos.data_ptr())
        s.region_off = self.region_off.ctypes.data
        s.cap = self.cap.ctypes.data
        s.len = self.len.ctypes.data

    def resized(self, caps, stream=None) -> "XkvCache":
        """The live tokens in a new cache whose streams have the capacities
        ``caps`` [L, B] (each >= the current length): xkv_repack, enqueued on the
        stream.  Used to leave the prompt-sized arena once the first eviction has
        shrunk every layer to its budget."""
        new = XkvCache(self.n_layers, self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim,
                       self.dtype, caps, device=self.k.device, zero=False)
        xkv_repack(self, new, 0, self.n_layers, stream=stream)
        return new

    def stream_slot(self, l, b, h) -> int:
        i = l * self.batch + b
        return int(self.region_off[i]) + h * int(self.cap[i])

    def length(self, l, b) -> int:
        return int(self.len[l * self.batch + b])


def xkv_workspace_bytes(cache: XkvCache, max_layers_per_call: int) -> int:
    out = C.c_size_t(0)
    _check(load().xkv_workspace_bytes(C.byref(cache.struct), int(max_layers_per_call), C.byref(out)),
           "xkv_workspace_bytes")
    return out.value


def xkv_decode_attend_score(cache: XkvCache, layer_begin, layer_end, q, k_new, v_new, pos_new,
                            out, workspace, softmax_scale: float = 0.0, stream=None):
    """q/k_new/v_new/out/workspace: torch device tensors; pos_new: int32 host array [B]."""
    pn = None if pos_new is None else np.ascontiguousarray(pos_new, dtype=np.int32)
    st = load().xkv_decode_attend_score(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(q), _ptr(k_new), _ptr(v_new),
        _ptr(pn), float(softmax_scale), _ptr(out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "xkv_decode_attend_score")


def xkv_decode_attend_score_noalloc(cache: XkvCache, layer_begin, layer_end, q, k_new, v_new, pos_new,
                                    out, softmax_scale: float = 0.0, stream=None):
    """The same call without a workspace: the library's fixed scratch array is used and nothing is allocated."""
    pn = None if pos_new is None else np.ascontiguousarray(pos_new, dtype=np.int32)
    st = load().xkv_decode_attend_score_noalloc(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(q), _ptr(k_new), _ptr(v_new),
        _ptr(pn), float(softmax_scale), _ptr(out), _stream_handle(stream))
    _check(st, "xkv_decode_attend_score_noalloc")


def xkv_decode_step(cache: XkvCache, layer_begin, layer_end, q, k_new, v_new, pos_new, out, budgets, workspace,
                    pool_size: int = 1, n_protect: int = 0, kept_idx_out=None, softmax_scale: float = 0.0,
                    stream=None):
    """xkv_decode_attend_score followed by xkv_evict_compact as one call."""
    pn = None if pos_new is None else np.ascontiguousarray(pos_new, dtype=np.int32)
    bud = None if budgets is None else np.ascontiguousarray(budgets, dtype=np.int32)
    st = load().xkv_decode_step(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(pn),
        float(softmax_scale), _ptr(out), _ptr(bud), int(pool_size), int(n_protect), _ptr(kept_idx_out),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream_handle(stream))
    _check(st, "xkv_decode_step")


def xkv_repack(src: XkvCache, dst: XkvCache, layer_begin, layer_end, stream=None):
    """Live tokens of src's layers into dst (same shape, other capacities); dst.len follows."""
    _check(load().xkv_repack(C.byref(src.struct), C.byref(dst.struct), int(layer_begin), int(layer_end),
                             _stream_handle(stream)), "xkv_repack")


def xkv_evict_compact(cache: XkvCache, layer_begin, layer_end, budgets, workspace, pool_size: int = 1,
                      n_protect: int = 0, kept_idx_out=None, stream=None):
    """budgets: int32 host array [layers, B]."""
    bud = None if budgets is None else np.ascontiguousarray(budgets, dtype=np.int32)
    st = load().xkv_evict_compact(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(bud), int(pool_size),
        int(n_protect), _ptr(kept_idx_out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "xkv_evict_compact")


def xkv_prefill_workspace_bytes(cache: XkvCache, max_layers_per_call: int, t: int, ows: int) -> int:
    out = C.c_size_t(0)
    _check(load().xkv_prefill_workspace_bytes(C.byref(cache.struct), int(max_layers_per_call), int(t),
                                              int(ows), C.byref(out)), "xkv_prefill_workspace_bytes")
    return out.value


def xkv_prefill_evict(cache: XkvCache, layer_begin, layer_end, q_win, k_src, v_src, t: int, ows: int,
                      budgets, workspace, pool_size: int = 1, softmax_scale: float = 0.0, w_out=None,
                      stream=None, t_per_seq=None):
    """q_win [layers, B, Hq, ows, d], k_src / v_src [layers, B, Hkv, t, d]: device tensors of the
    cache dtype; budgets: int32 host array [layers, B]; w_out: device fp32 [layers, B, Hkv, t] or None."""
    bud = None if budgets is None else np.ascontiguousarray(budgets, dtype=np.int32)
    tps = None if t_per_seq is None else np.ascontiguousarray(t_per_seq, dtype=np.int32)
    st = load().xkv_prefill_evict(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(q_win), _ptr(k_src), _ptr(v_src),
        int(t), _ptr(tps), int(ows), int(pool_size), _ptr(bud), float(softmax_scale), _ptr(w_out),
        _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "xkv_prefill_evict")


def xkv_prefill_evict_lse(cache: XkvCache, layer_begin, layer_end, q_win, k_src, v_src, t: int, ows: int,
                          budgets, lse_win, workspace, pool_size: int = 1, softmax_scale: float = 0.0, w_out=None,
                          stream=None, t_per_seq=None):
    """xkv_prefill_evict with the window rows' normalisers given: lse_win device fp32 [layers, B, Hq, ows]."""
    bud = None if budgets is None else np.ascontiguousarray(budgets, dtype=np.int32)
    tps = None if t_per_seq is None else np.ascontiguousarray(t_per_seq, dtype=np.int32)
    st = load().xkv_prefill_evict_lse(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(q_win), _ptr(k_src), _ptr(v_src),
        int(t), _ptr(tps), int(ows), int(pool_size), _ptr(bud), float(softmax_scale), _ptr(lse_win), _ptr(w_out),
        _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "xkv_prefill_evict_lse")


def xkv_window_importance_lse(cache: XkvCache, layer_begin, layer_end, q_win, k_src, t: int, ows: int, lse_win,
                              w_out, workspace, pool_size: int = 1, softmax_scale: float = 0.0, stream=None,
                              t_per_seq=None):
    """xkv_window_importance with the window rows' normalisers given: lse_win device fp32 [layers, B, Hq, ows]."""
    tps = None if t_per_seq is None else np.ascontiguousarray(t_per_seq, dtype=np.int32)
    st = load().xkv_window_importance_lse(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(q_win), _ptr(k_src), int(t), _ptr(tps),
        int(ows), int(pool_size), float(softmax_scale), _ptr(lse_win), _ptr(w_out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "xkv_window_importance_lse")


def xkv_window_importance(cache: XkvCache, layer_begin, layer_end, q_win, k_src, t: int, ows: int, w_out,
                          workspace, pool_size: int = 1, softmax_scale: float = 0.0, stream=None,
                          t_per_seq=None):
    """w_out: device fp32 [layers, B, t - ows], the per-(layer, sequence) score distribution vectors."""
    tps = None if t_per_seq is None else np.ascontiguousarray(t_per_seq, dtype=np.int32)
    st = load().xkv_window_importance(
        C.byref(cache.struct), int(layer_begin), int(layer_end), _ptr(q_win), _ptr(k_src), int(t), _ptr(tps),
        int(ows), int(pool_size), float(softmax_scale), _ptr(w_out), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "xkv_window_importance")


def xkv_cache_importance(cache: XkvCache, layer_begin, layer_end, n_pos: int, w_out, stream=None):
    """w_out: device fp32 [layers, B, n_pos]: the position-indexed score vector of every (layer, sequence)."""
    _check(load().xkv_cache_importance(C.byref(cache.struct), int(layer_begin), int(layer_end), int(n_pos),
                                       _ptr(w_out), _stream_handle(stream)), "xkv_cache_importance")


def xkv_allocate_device_workspace_bytes(n_layers: int, length: int) -> int:
    out = C.c_size_t(0)
    _check(load().xkv_allocate_device_workspace_bytes(int(n_layers), int(length), C.byref(out)),
           "xkv_allocate_device_workspace_bytes")
    return out.value


def xkv_allocate_budgets_device(w, n_layers: int, length: int, layer_stride: int, total_size: int, workspace,
                                min_budget=None, max_budget=None, stream=None, mode: int = XKV_ALLOC_TOTAL_SIZE,
                                target_ravg: float = 0.0):
    """w: device fp32 tensor; layer l's `length` values start at element l * layer_stride of it.
    Returns (budgets int64 [n_layers], R_avg).  Waits for the stream."""
    lo = None if min_budget is None else np.ascontiguousarray(min_budget, dtype=np.int64)
    hi = None if max_budget is None else np.ascontiguousarray(max_budget, dtype=np.int64)
    out = np.zeros(int(n_layers), dtype=np.int64)
    ravg = C.c_double(0.0)
    st = load().xkv_allocate_budgets_device(
        int(n_layers), _ptr(w), int(length), int(layer_stride), int(mode), int(total_size), float(target_ravg),
        _ptr(lo), _ptr(hi),
        out.ctypes.data, C.byref(ravg), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    _check(st, "xkv_allocate_budgets_device")
    return out, ravg.value


def xkv_configure(key: int, value: int):
    _check(load().xkv_configure(int(key), int(value)), "xkv_configure")


def xkv_fused_status() -> bool:
    """True if a launch of the most recent fused decode call gave up its grid-wide wait.  Waits for its stream."""
    flag = C.c_int32(0)
    _check(load().xkv_fused_status(C.byref(flag)), "xkv_fused_status")
    return bool(flag.value)


def xkv_probe_stream_read(buffer, non_temporal: bool, store_floats_per_workgroup: int = 0, sink=None,
                          stream=None, store_policy: int = 2):
    """One launch of the read-only streaming kernel over a torch device tensor."""
    _check(load().xkv_probe_stream_read(_ptr(buffer), buffer.numel() * buffer.element_size(),
                                        1 if non_temporal else 0, int(store_floats_per_workgroup),
                                        int(store_policy), _ptr(sink), _stream_handle(stream)),
           "xkv_probe_stream_read")


def xkv_profile_enable(on: bool):
    _check(load().xkv_profile_enable(1 if on else 0), "xkv_profile_enable")


def xkv_profile_read(kernel_index: int):
    n, ms = C.c_int64(0), C.c_double(0.0)
    _check(load().xkv_profile_read(int(kernel_index), C.byref(n), C.byref(ms)), "xkv_profile_read")
    return n.value, ms.value
