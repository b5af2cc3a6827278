from __future__ import annotations

import ctypes
import os

import torch

__all__ = [
    "SkvError", "Cache", "lib", "SKV_F32", "SKV_F16", "SKV_BF16", "SKV_BF16_KV8", "SKV_F16_KV8", "STATUS", "dtype_code",
    "skv_cache_pool_bytes", "skv_cache_scale_info", "skv_cache_set_eviction",
    "skv_route_from_strategy", "skv_route_validate", "skv_cache_bytes", "skv_cache_alloc",
    "skv_cache_free", "skv_cache_info", "skv_cache_slot_of_layer", "skv_cache_set_block_table",
    "skv_cache_device_faults", "skv_kv_append", "skv_kv_project_append", "skv_kv_project_workspace_bytes", "skv_decode_workspace_bytes", "skv_attn_decode",
    "skv_decode_range_workspace_bytes", "skv_attn_decode_range", "skv_static_scratch_bytes", "skv_attn_decode_static", "skv_attn_prefill", "skv_status_str", "skv_last_hip_error", "skv_last_kernel_name",
    "skv_train_sample_route", "skv_train_attn_fwd", "skv_train_bwd_workspace_bytes",
    "skv_train_attn_bwd", "skv_train_device_faults", "SKV_TRAIN_RCLA", "SKV_TRAIN_CLA_K", "SKV_TRAIN_RDCLA_K",
]

SKV_F32, SKV_F16, SKV_BF16, SKV_BF16_KV8, SKV_F16_KV8 = 0, 1, 2, 3, 4
SKV_TRAIN_RCLA, SKV_TRAIN_CLA_K, SKV_TRAIN_RDCLA_K = 0, 1, 2
STATUS = {0: "SKV_OK", 1: "SKV_ERR_INVALID_ARG", 2: "SKV_ERR_BAD_ROUTE", 3: "SKV_ERR_NOT_OWNER",
          4: "SKV_ERR_CAPACITY", 5: "SKV_ERR_OOM", 6: "SKV_ERR_UNSUPPORTED", 7: "SKV_ERR_HIP"}

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libskv.so")
_lib = None


class SkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)}")


class _Desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "n_q_heads", "n_kv_heads", "head_dim", "batch", "max_ctx", "dtype",
                 "block_size", "n_blocks")] + [
        ("route", ctypes.POINTER(ctypes.c_int32)), ("k_pool", ctypes.c_void_p),
        ("v_pool", ctypes.c_void_p), ("pool_bytes", ctypes.c_size_t),
        ("scale_pool", ctypes.c_void_p), ("scale_pool_bytes", ctypes.c_size_t)]


def lib() -> ctypes.CDLL:
    """The loaded HIP library.  Built in-tree first if (and only if) no built library exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from .build import build_library
            build_library()
        L = ctypes.CDLL(_LIB_PATH)
        for name in __all__:
            if name.startswith("skv_"):
                getattr(L, name).restype = ctypes.c_int32
        L.skv_status_str.restype = ctypes.c_char_p
        L.skv_last_kernel_name.restype = ctypes.c_char_p
        _lib = L
    return _lib


def dtype_code(dt: torch.dtype, kv8: bool = False) -> int:
    """Descriptor dtype of a cache whose queries / new rows / outputs have torch dtype dt; kv8: 8-bit slots."""
    if kv8:
        return {torch.float16: SKV_F16_KV8, torch.bfloat16: SKV_BF16_KV8}[dt]
    return {torch.float32: SKV_F32, torch.float16: SKV_F16, torch.bfloat16: SKV_BF16}[dt]


def _check(st: int, where: str):
    if st != 0:
        raise SkvError(st, where)


def _i32(values):
    arr = (ctypes.c_int32 * len(values))(*[int(v) for v in values])
    return arr


def _ptr(t):
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    assert t.is_contiguous(), "skv takes dense tensors"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    return ctypes.c_void_p(stream)


def _desc(n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_ctx, dtype, route, block_size=0,
          n_blocks=0, k_pool=None, v_pool=None, pool_bytes=0, scale_pool=None, scale_pool_bytes=0):
    route_arr = _i32(route) if route is not None else None
    d = _Desc(n_layers, n_q_heads, n_kv_heads, head_dim, batch, max_ctx, dtype, block_size, n_blocks,
              ctypes.cast(route_arr, ctypes.POINTER(ctypes.c_int32)) if route_arr is not None else None,
              _ptr(k_pool), _ptr(v_pool), pool_bytes, _ptr(scale_pool), scale_pool_bytes)
    d._keep = (route_arr, k_pool, v_pool, scale_pool)
    return d


class Cache:
    """Owner of a skv_cache_t*.  Keeps borrowed tensors (pools, block table) alive."""

    def __init__(self, handle, keep):
        self.handle = handle
        self._keep = list(keep)

    def free(self):
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().skv_cache_free(h), "skv_cache_free")

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def skv_route_from_strategy(owners, n_layers):
    out = (ctypes.c_int32 * max(n_layers, 1))()
    _check(lib().skv_route_from_strategy(_i32(owners), len(owners), n_layers, out), "skv_route_from_strategy")
    return list(out)[:n_layers]


def skv_route_validate(route):
    """-> (slot_of_layer, n_slots)"""
    n = len(route)
    slot = (ctypes.c_int32 * max(n, 1))()
    ns = ctypes.c_int32(0)
    _check(lib().skv_route_validate(_i32(route), n, slot, ctypes.byref(ns)), "skv_route_validate")
    return list(slot)[:n], ns.value


def skv_cache_bytes(**desc):
    d = _desc(**desc)
    out = ctypes.c_size_t(0)
    _check(lib().skv_cache_bytes(ctypes.byref(d), ctypes.byref(out)), "skv_cache_bytes")
    return out.value


def skv_cache_pool_bytes(**desc):
    """-> (bytes of the K pool (= of the V pool), bytes of the pool of exponent bytes)"""
    d = _desc(**desc)
    kv, sc = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().skv_cache_pool_bytes(ctypes.byref(d), ctypes.byref(kv), ctypes.byref(sc)), "skv_cache_pool_bytes")
    return kv.value, sc.value


def skv_cache_scale_info(cache: "Cache"):
    """-> (scale_pool_ptr, scale_pool_bytes)"""
    sp, sb = ctypes.c_void_p(0), ctypes.c_size_t(0)
    _check(lib().skv_cache_scale_info(cache.handle, ctypes.byref(sp), ctypes.byref(sb)), "skv_cache_scale_info")
    return sp.value, sb.value


def skv_cache_alloc(**desc) -> Cache:
    d = _desc(**desc)
    h = ctypes.c_void_p(0)
    _check(lib().skv_cache_alloc(ctypes.byref(d), ctypes.byref(h)), "skv_cache_alloc")
    return Cache(h, [desc.get("k_pool"), desc.get("v_pool"), desc.get("scale_pool")])


def skv_cache_free(cache: Cache):
    cache.free()


def skv_cache_info(cache: Cache):
    """-> (n_slots, k_pool_ptr, v_pool_ptr, pool_bytes_each)"""
    ns, kp, vp, pb = ctypes.c_int32(0), ctypes.c_void_p(0), ctypes.c_void_p(0), ctypes.c_size_t(0)
    _check(lib().skv_cache_info(cache.handle, ctypes.byref(ns), ctypes.byref(kp), ctypes.byref(vp),
                                ctypes.byref(pb)), "skv_cache_info")
    return ns.value, kp.value, vp.value, pb.value


def skv_cache_slot_of_layer(cache: Cache, layer: int):
    """-> (slot, is_owner)"""
    s, o = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().skv_cache_slot_of_layer(cache.handle, layer, ctypes.byref(s), ctypes.byref(o)),
           "skv_cache_slot_of_layer")
    return s.value, bool(o.value)


def skv_cache_set_block_table(cache: Cache, table: torch.Tensor):
    assert table.dtype == torch.int32 and table.dim() == 2
    _check(lib().skv_cache_set_block_table(cache.handle, _ptr(table), table.shape[1]),
           "skv_cache_set_block_table")
    cache._keep.append(table)


def skv_cache_set_eviction(cache: Cache, sink_len, first_pos):
    """sink_len, first_pos: int32 device tensors [batch], or both None to switch eviction off."""
    if sink_len is not None:
        assert sink_len.dtype == torch.int32 and first_pos.dtype == torch.int32
    _check(lib().skv_cache_set_eviction(cache.handle, _ptr(sink_len), _ptr(first_pos)), "skv_cache_set_eviction")
    cache._evict = (sink_len, first_pos)


def skv_cache_device_faults(cache: Cache) -> int:
    f = ctypes.c_uint32(0)
    _check(lib().skv_cache_device_faults(cache.handle, ctypes.byref(f)), "skv_cache_device_faults")
    return f.value


def skv_kv_append(cache: Cache, layer: int, k_new, v_new, start_pos, new_lens, max_new: int, stream=None):
    _check(lib().skv_kv_append(cache.handle, layer, _ptr(k_new), _ptr(v_new), _ptr(start_pos),
                               _ptr(new_lens), max_new, _stream(stream)), "skv_kv_append")


def skv_kv_project_workspace_bytes(cache: Cache, max_new: int, hidden: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().skv_kv_project_workspace_bytes(cache.handle, max_new, hidden, ctypes.byref(out)),
           "skv_kv_project_workspace_bytes")
    return out.value


def skv_kv_project_append(cache: Cache, layer: int, x, w_k, w_v, rope_cos, rope_sin, start_pos, new_lens,
                          max_new: int, workspace=None, stream=None, k_norm_weight=None, k_norm_eps: float = 1e-6):
    """x: [batch][max_new][hidden]; w_k, w_v: [n_kv_heads * head_dim][hidden]; rope_cos, rope_sin:
    float32 [positions][head_dim / 2] or None; k_norm_weight: float32 [head_dim] or None."""
    if k_norm_weight is not None and k_norm_weight.dtype != torch.float32:
        raise ValueError("k_norm_weight is float32 [head_dim]")
    hidden = x.shape[-1]
    if w_k.shape[-1] != hidden or w_v.shape[-1] != hidden or w_k.dtype != x.dtype or w_v.dtype != x.dtype:
        raise ValueError("w_k and w_v are [n_kv_heads * head_dim][hidden] in the dtype of x")
    n_pos = 0
    if rope_cos is not None:
        if rope_cos.dtype != torch.float32 or rope_sin.dtype != torch.float32 or rope_cos.shape != rope_sin.shape:
            raise ValueError("rope tables are float32 [positions][head_dim / 2]")
        n_pos = rope_cos.shape[0]
    wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().skv_kv_project_append(cache.handle, layer, _ptr(x), _ptr(w_k), _ptr(w_v), _ptr(rope_cos),
                                       _ptr(rope_sin), n_pos, _ptr(k_norm_weight), ctypes.c_float(k_norm_eps),
                                       _ptr(start_pos), _ptr(new_lens), max_new, hidden,
                                       _ptr(workspace), ctypes.c_size_t(wb), _stream(stream)), "skv_kv_project_append")


def skv_decode_workspace_bytes(cache: Cache, max_kv_len: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().skv_decode_workspace_bytes(cache.handle, max_kv_len, ctypes.byref(out)),
           "skv_decode_workspace_bytes")
    return out.value


def skv_attn_decode(cache: Cache, layer: int, q, out, kv_lens, max_kv_len: int, scale: float,
                    workspace, stream=None):
    wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().skv_attn_decode(cache.handle, layer, _ptr(q), _ptr(out), _ptr(kv_lens), max_kv_len,
                                 ctypes.c_float(scale), _ptr(workspace), ctypes.c_size_t(wb),
                                 _stream(stream)), "skv_attn_decode")


def skv_decode_range_workspace_bytes(cache: Cache, seq_count: int, max_kv_len: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().skv_decode_range_workspace_bytes(cache.handle, seq_count, max_kv_len, ctypes.byref(out)),
           "skv_decode_range_workspace_bytes")
    return out.value


def skv_attn_decode_range(cache: Cache, layer: int, seq_begin: int, seq_count: int, q, out, kv_lens,
                          max_kv_len: int, scale: float, workspace, stream=None):
    """q, out, kv_lens: tensors (views) that start at the first sequence of the range."""
    wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().skv_attn_decode_range(cache.handle, layer, seq_begin, seq_count, _ptr(q), _ptr(out),
                                       _ptr(kv_lens), max_kv_len, ctypes.c_float(scale), _ptr(workspace),
                                       ctypes.c_size_t(wb), _stream(stream)), "skv_attn_decode_range")


def skv_static_scratch_bytes() -> int:
    out = ctypes.c_size_t(0)
    _check(lib().skv_static_scratch_bytes(ctypes.byref(out)), "skv_static_scratch_bytes")
    return out.value


def skv_attn_decode_static(cache: Cache, layer: int, q, out, kv_lens, max_kv_len: int, scale: float, stream=None):
    _check(lib().skv_attn_decode_static(cache.handle, layer, _ptr(q), _ptr(out), _ptr(kv_lens), max_kv_len,
                                        ctypes.c_float(scale), _stream(stream)), "skv_attn_decode_static")


def skv_attn_prefill(cache: Cache, layer: int, q, out, q_lens, kv_lens, max_q: int, max_kv_len: int,
                     scale: float, stream=None):
    _check(lib().skv_attn_prefill(cache.handle, layer, _ptr(q), _ptr(out), _ptr(q_lens), _ptr(kv_lens),
                                  max_q, max_kv_len, ctypes.c_float(scale), _stream(stream)),
           "skv_attn_prefill")


def skv_train_sample_route(scheme: int, n_layers: int, k: int, p: float, seed: int, step: int) -> list:
    route = (ctypes.c_int32 * max(n_layers, 1))()
    _check(lib().skv_train_sample_route(scheme, n_layers, k, ctypes.c_double(p), ctypes.c_uint64(seed),
                                        ctypes.c_uint64(step), route), "skv_train_sample_route")
    return list(route)[:n_layers]


def _train_shapes(q, k):
    batch, seq, hq, d = q.shape
    if k.shape[0] != batch or k.shape[1] != seq or k.shape[3] != d:
        raise ValueError("q is [batch][seq][n_q_heads][head_dim], k and v [batch][seq][n_kv_heads][head_dim]")
    return batch, seq, hq, k.shape[2], d


def skv_train_attn_fwd(q, k, v, out, lse, seq_lens, scale: float, stream=None):
    """q, out: [batch][seq][n_q_heads][head_dim]; k, v: [batch][seq][n_kv_heads][head_dim];
    lse: float32 [batch][n_q_heads][seq]; seq_lens: int32 [batch] (all device tensors)."""
    batch, seq, hq, hkv, d = _train_shapes(q, k)
    _check(lib().skv_train_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(seq_lens), batch, seq,
                                    hq, hkv, d, dtype_code(q.dtype), ctypes.c_float(scale), _stream(stream)),
           "skv_train_attn_fwd")


def skv_train_bwd_workspace_bytes(batch: int, seq: int, n_q_heads: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().skv_train_bwd_workspace_bytes(batch, seq, n_q_heads, ctypes.byref(out)),
           "skv_train_bwd_workspace_bytes")
    return out.value


def skv_train_attn_bwd(q, k, v, out, lse, d_out, dq, dk_accum, dv_accum, seq_lens, scale: float, workspace,
                       stream=None):
    """dk_accum, dv_accum: float32 tensors of the shape of k; the gradients are ADDED to them."""
    batch, seq, hq, hkv, d = _train_shapes(q, k)
    if dk_accum.dtype != torch.float32 or dv_accum.dtype != torch.float32 or lse.dtype != torch.float32:
        raise ValueError("lse, dk_accum and dv_accum are float32")
    wb = workspace.numel() * workspace.element_size()
    _check(lib().skv_train_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(d_out), _ptr(dq),
                                    _ptr(dk_accum), _ptr(dv_accum), _ptr(seq_lens), batch, seq, hq, hkv, d,
                                    dtype_code(q.dtype), ctypes.c_float(scale), _ptr(workspace),
                                    ctypes.c_size_t(wb), _stream(stream)), "skv_train_attn_bwd")


def skv_train_device_faults() -> int:
    out = ctypes.c_uint32(0)
    _check(lib().skv_train_device_faults(ctypes.byref(out)), "skv_train_device_faults")
    return out.value


def skv_status_str(status: int) -> str:
    return lib().skv_status_str(status).decode()


def skv_last_hip_error() -> int:
    return lib().skv_last_hip_error()


def skv_last_kernel_name() -> str:
    return lib().skv_last_kernel_name().decode()
