"""ctypes binding of libellm.so: the functions of include/ellm.h under the same names.

Argument marshalling only. Device buffers are passed as torch tensors (or raw integer addresses),
host arrays as numpy arrays or sequences; a negative return code raises EllmError carrying the
code, unless `check=False` is given, in which case the code is returned.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libellm.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
        "or python paper_2506_15155_amd/build.py). There is no fallback implementation.")

lib = C.CDLL(LIB_PATH)

ELLM_OWNER_KV, ELLM_OWNER_ACT = 0, 1
ELLM_CHUNK_FREE, ELLM_CHUNK_MAPPED, ELLM_CHUNK_BUSY = 0, 1, 2
ELLM_BF16 = 1
ELLM_MAP_ALLOW_INFLATE = 1
ELLM_POOL_METADATA_ONLY = 1
ELLM_POOL_DRIVER_MAPPED = 2
ELLM_NOALLOC_WORKSPACE_BYTES = 16 << 20


class ERR:
    OK, INVALID, OOM, OWNED, UNMAPPED, NOT_RESIDENT, RANGE, EMPTY, HOST_FULL, HIP, NO_DEVICE = (
        0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10)


class EllmError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libellm error {code}: {text}")
        self.code = code


class _Desc(C.Structure):
    _fields_ = [("device_base", C.c_void_p), ("device_bytes", C.c_uint64),
                ("host_base", C.c_void_p), ("host_bytes", C.c_uint64),
                ("chunk_bytes", C.c_uint32),
                ("n_q_heads", C.c_uint16), ("n_kv_heads", C.c_uint16), ("head_dim", C.c_uint16), ("dtype", C.c_uint16),
                ("max_tensors", C.c_uint32), ("max_slots_per_tensor", C.c_uint32),
                ("flags", C.c_uint32), ("reserved", C.c_uint32),
                ("initial_owner", C.c_void_p)]


_i32p = C.POINTER(C.c_int32)
_vp = C.c_void_p
_sigs = {
    "ellm_pool_create": [C.POINTER(_Desc), C.POINTER(_vp)],
    "ellm_pool_destroy": [_vp],
    "ellm_tensor_create": [_vp, C.c_int64, _i32p],
    "ellm_tensor_destroy": [_vp, C.c_int32],
    "ellm_tensor_release": [_vp, C.c_int32],
    "ellm_tensor_acquire": [_vp, C.c_int64, C.c_int64, C.c_uint32, _i32p],
    "ellm_tensor_is_released": [_vp, C.c_int32],
    "ellm_kv_premap_next": [_vp, _i32p, C.c_int32, C.c_uint32, _i32p],
    "ellm_kv_premap_ahead": [_vp, _i32p, C.c_int32, C.c_int64, C.c_uint32, _i32p],
    "ellm_pool_flush_tables": [_vp, _vp],
    "ellm_pool_set_logical_host_slots": [_vp, C.c_int32],
    "ellm_pool_get_logical_host_slots": [_vp, _i32p],
    "ellm_pool_slo_configure": [_vp, C.c_double, C.c_double, C.c_double, C.c_int32, C.c_int32],
    "ellm_pool_slo_observe": [_vp, C.c_double, C.c_double, _i32p],
    "ellm_debug_vmm_buffer_create": [C.c_uint64, C.c_int32, C.c_uint32, C.c_uint16, C.POINTER(C.c_void_p), C.POINTER(C.c_uint64)],
    "ellm_debug_vmm_buffer_destroy": [_vp],
    "ellm_debug_vmm_latency": [C.c_uint64, C.c_int32, C.POINTER(C.c_double)],
    "ellm_tensor_map_chunks": [_vp, C.c_int32, C.c_int32, C.c_int32, _i32p, C.c_uint32],
    "ellm_tensor_unmap_chunks": [_vp, C.c_int32, C.c_int32, C.c_int32],
    "ellm_pool_transfer": [_vp, _i32p, C.c_int32, C.c_int],
    "ellm_pool_set_act_busy": [_vp, _i32p, C.c_int32, C.c_int],
    "ellm_kv_append": [_vp, _i32p, C.c_int32, _i32p, _vp, _vp, _vp],
    "ellm_decode_attention": [_vp, _i32p, C.c_int32, _vp, _vp, C.c_float, _vp],
    "ellm_decode_attention_noalloc": [_vp, _i32p, C.c_int32, _vp, _vp, C.c_float, _vp],
    "ellm_kv_append_decode": [_vp, _i32p, C.c_int32, _vp, _vp, _vp, _vp, C.c_float, _vp],
    "ellm_chunk_deflate_to_host": [_vp, C.c_int32, C.c_int32, C.c_int32],
    "ellm_chunk_inflate_from_host": [_vp, C.c_int32, C.c_int32, C.c_int32, _i32p],
    "ellm_pool_sync": [_vp],
    "ellm_pool_prepare": [_vp, _vp],
    "ellm_debug_fail_launch": [_vp, C.c_int32],
    "ellm_pool_get_device_base": [_vp, C.POINTER(C.c_void_p)],
    "ellm_pool_get_mapping_stats": [_vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)],
    "ellm_debug_set_table_kernels": [_vp, C.c_int],
    "ellm_debug_set_async_mapping": [_vp, C.c_int],
    "ellm_debug_set_copy_kernels": [_vp, C.c_int],
    "ellm_debug_fail_mapping": [_vp, C.c_int32],
    "ellm_pool_get_mapping_wait": [_vp, C.POINTER(C.c_double)],
    "ellm_pool_get_geometry": [_vp, _i32p, _i32p, _i32p, C.POINTER(C.c_uint64)],
    "ellm_tensor_get_table": [_vp, C.c_int32, _i32p, C.c_int32, _i32p, C.POINTER(C.c_int64)],
    "ellm_pool_get_owner_state": [_vp, _vp, _vp, _i32p, _i32p],
    "ellm_pool_get_host_slots": [_vp, _i32p, _i32p],
    "ellm_decode_plan": [_vp, _i32p, C.c_int32, _i32p, _i32p],
    "ellm_pool_set_split_tokens": [_vp, C.c_int32],
    "ellm_pool_self_check": [_vp],
    "ellm_debug_set_waves": [_vp, C.c_int32],
    "ellm_debug_copy": [_vp, _vp, C.c_uint64, _vp],
    "ellm_debug_stream_read": [_vp, C.c_uint64, _vp, _vp],
    "ellm_debug_kv_stream_read": [_vp, _i32p, C.c_int32, _vp, _vp],
    "ellm_pool_profile_stride": [_vp, C.c_int32],
    "ellm_pool_profile_enable": [_vp, C.c_int32],
    "ellm_pool_profile_collect": [_vp, C.POINTER(C.c_float), C.c_int32, _i32p],
}
for _n, _a in _sigs.items():
    getattr(lib, _n).argtypes = _a
    getattr(lib, _n).restype = C.c_int
lib.ellm_last_error.restype = C.c_char_p
lib.ellm_last_error.argtypes = []
lib.ellm_workspace_bytes.restype = C.c_uint64
lib.ellm_workspace_bytes.argtypes = [C.POINTER(_Desc), C.c_int32]

EXPORTED = sorted(list(_sigs) + ["ellm_last_error", "ellm_workspace_bytes"])


def ellm_last_error() -> str:
    return lib.ellm_last_error().decode()


def _ret(rc: int, check: bool):
    if rc < 0 and check:
        raise EllmError(rc, ellm_last_error())
    return rc


def _ptr(x) -> int | None:
    """Device or host address of a torch tensor / numpy array / int."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError(type(x))


def _i32(a):
    if a is None:
        return None, None, 0
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(_i32p), arr.size


def _stream(stream) -> int | None:
    """hipStream_t of a torch stream (or a raw handle). None selects torch's current stream."""
    if stream is None:
        import torch
        if not torch.cuda.is_available():
            return None
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def ellm_pool_create(device_buf, host_buf, chunk_bytes, n_q_heads, n_kv_heads, head_dim, max_tensors,
                     max_slots_per_tensor, initial_owner=None, flags=0, device_bytes=None, host_bytes=None,
                     check=True):
    """device_buf / host_buf: torch uint8 tensors (device / pinned host), or None. Returns the pool
    handle (an int); with check=False returns (rc, handle)."""
    d = _Desc()
    d.device_base = _ptr(device_buf)
    d.device_bytes = device_bytes if device_bytes is not None else (device_buf.numel() * device_buf.element_size()
                                                                     if device_buf is not None else 0)
    d.host_base = _ptr(host_buf)
    d.host_bytes = host_bytes if host_bytes is not None else (host_buf.numel() * host_buf.element_size()
                                                               if host_buf is not None else 0)
    d.chunk_bytes, d.n_q_heads, d.n_kv_heads, d.head_dim, d.dtype = chunk_bytes, n_q_heads, n_kv_heads, head_dim, ELLM_BF16
    d.max_tensors, d.max_slots_per_tensor, d.flags, d.reserved = max_tensors, max_slots_per_tensor, flags, 0
    own = None
    if initial_owner is not None:
        own = np.ascontiguousarray(initial_owner, dtype=np.uint8)
        d.initial_owner = own.ctypes.data
    out = _vp()
    rc = lib.ellm_pool_create(C.byref(d), C.byref(out))
    if check:
        _ret(rc, True)
        return out.value
    return rc, out.value


def ellm_pool_destroy(pool, check=True):
    return _ret(lib.ellm_pool_destroy(pool), check)


def ellm_tensor_create(pool, max_tokens, check=True):
    out = C.c_int32(-1)
    rc = lib.ellm_tensor_create(pool, int(max_tokens), C.byref(out))
    if check:
        _ret(rc, True)
        return out.value
    return rc, out.value


def ellm_tensor_destroy(pool, tid, check=True):
    return _ret(lib.ellm_tensor_destroy(pool, tid), check)


def ellm_tensor_release(pool, tid, check=True):
    return _ret(lib.ellm_tensor_release(pool, tid), check)


def ellm_tensor_acquire(pool, need_tokens, max_tokens, flags=0, check=True):
    """Returns the handle (check=True) or (rc, handle)."""
    out = C.c_int32(-1)
    rc = lib.ellm_tensor_acquire(pool, int(need_tokens), int(max_tokens), int(flags), C.byref(out))
    if check:
        _ret(rc, True)
        return out.value
    return rc, out.value


def ellm_tensor_is_released(pool, tid):
    return lib.ellm_tensor_is_released(pool, tid)


def ellm_kv_premap_ahead(pool, ids, tokens_ahead, flags=0, check=True):
    """Returns the number of chunks mapped (check=True) or (rc, n)."""
    _, p, n = _i32(ids)
    out = C.c_int32(0)
    rc = lib.ellm_kv_premap_ahead(pool, p, n, int(tokens_ahead), int(flags), C.byref(out))
    if check:
        _ret(rc, True)
        return out.value
    return rc, out.value


def ellm_kv_premap_next(pool, ids, flags=0, check=True):
    """Returns the number of chunks mapped (check=True) or (rc, n)."""
    _, p, n = _i32(ids)
    out = C.c_int32(0)
    rc = lib.ellm_kv_premap_next(pool, p, n, int(flags), C.byref(out))
    if check:
        _ret(rc, True)
        return out.value
    return rc, out.value


def ellm_pool_flush_tables(pool, stream=None, check=True):
    return _ret(lib.ellm_pool_flush_tables(pool, _stream(stream)), check)


def ellm_pool_set_logical_host_slots(pool, n, check=True):
    return _ret(lib.ellm_pool_set_logical_host_slots(pool, int(n)), check)


def ellm_pool_get_logical_host_slots(pool):
    out = C.c_int32(0)
    _ret(lib.ellm_pool_get_logical_host_slots(pool, C.byref(out)), True)
    return out.value


def ellm_pool_slo_configure(pool, ttft_slo, tpot_slo, alpha=2.0, window=5, threshold=3, check=True):
    return _ret(lib.ellm_pool_slo_configure(pool, float(ttft_slo), float(tpot_slo), float(alpha), int(window),
                                            int(threshold)), check)


def ellm_pool_slo_observe(pool, ttft, tpot, check=True):
    """Returns the logical size after the call (check=True) or (rc, size)."""
    out = C.c_int32(0)
    rc = lib.ellm_pool_slo_observe(pool, float(ttft), float(tpot), C.byref(out))
    if check:
        _ret(rc, True)
        return out.value
    return rc, out.value


def ellm_debug_vmm_buffer_create(chunk_bytes, n_chunks, seed=0, fill16=0, check=True):
    """Returns (base address, bytes); with check=False (rc, base, bytes)."""
    base, nbytes = C.c_void_p(), C.c_uint64()
    rc = lib.ellm_debug_vmm_buffer_create(int(chunk_bytes), int(n_chunks), int(seed), int(fill16), C.byref(base),
                                          C.byref(nbytes))
    if check:
        _ret(rc, True)
        return int(base.value), int(nbytes.value)
    return rc, int(base.value or 0), int(nbytes.value)


def ellm_debug_vmm_buffer_destroy(base, check=True):
    return _ret(lib.ellm_debug_vmm_buffer_destroy(int(base)), check)


def ellm_debug_vmm_latency(chunk_bytes, n_chunks, check=True):
    """Host microseconds per chunk: (create, map + set-access, unmap, release)."""
    us = (C.c_double * 4)()
    rc = lib.ellm_debug_vmm_latency(int(chunk_bytes), int(n_chunks), us)
    if check:
        _ret(rc, True)
        return tuple(us)
    return rc, tuple(us)


def ellm_tensor_map_chunks(pool, tid, first_slot, n_slots, chunk_ids=None, flags=0, check=True):
    _, p, _ = _i32(chunk_ids)
    return _ret(lib.ellm_tensor_map_chunks(pool, tid, first_slot, n_slots, p, flags), check)


def ellm_tensor_unmap_chunks(pool, tid, first_slot, n_slots, check=True):
    return _ret(lib.ellm_tensor_unmap_chunks(pool, tid, first_slot, n_slots), check)


def ellm_pool_transfer(pool, chunk_ids, new_owner, check=True):
    _, p, n = _i32(chunk_ids)
    return _ret(lib.ellm_pool_transfer(pool, p, n, new_owner), check)


def ellm_pool_set_act_busy(pool, chunk_ids, busy, check=True):
    _, p, n = _i32(chunk_ids)
    return _ret(lib.ellm_pool_set_act_busy(pool, p, n, int(busy)), check)


def ellm_kv_append(pool, ids, k_new, v_new, n_new=None, stream=None, check=True):
    _, p, n = _i32(ids)
    _, pn, _ = _i32(n_new)
    s = _stream(stream)
    return _ret(lib.ellm_kv_append(pool, p, n, pn, _ptr(k_new), _ptr(v_new), s), check)


def ellm_decode_attention(pool, ids, q, out, scale=0.0, stream=None, check=True):
    _, p, n = _i32(ids)
    s = _stream(stream)
    return _ret(lib.ellm_decode_attention(pool, p, n, _ptr(q), _ptr(out), float(scale), s), check)


def ellm_decode_attention_noalloc(pool, ids, q, out, scale=0.0, stream=None, check=True):
    _, p, n = _i32(ids)
    s = _stream(stream)
    return _ret(lib.ellm_decode_attention_noalloc(pool, p, n, _ptr(q), _ptr(out), float(scale), s), check)


def ellm_kv_append_decode(pool, ids, k_new, v_new, q, out, scale=0.0, stream=None, check=True):
    _, p, n = _i32(ids)
    return _ret(lib.ellm_kv_append_decode(pool, p, n, _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(out), float(scale),
                                          _stream(stream)), check)


def ellm_chunk_deflate_to_host(pool, tid, first_slot, n_slots, check=True):
    return _ret(lib.ellm_chunk_deflate_to_host(pool, tid, first_slot, n_slots), check)


def ellm_chunk_inflate_from_host(pool, tid, first_slot, n_slots, chunk_ids=None, check=True):
    _, p, _ = _i32(chunk_ids)
    return _ret(lib.ellm_chunk_inflate_from_host(pool, tid, first_slot, n_slots, p), check)


def ellm_pool_sync(pool, check=True):
    return _ret(lib.ellm_pool_sync(pool), check)


def ellm_pool_prepare(pool, stream=None, check=True):
    return _ret(lib.ellm_pool_prepare(pool, _stream(stream)), check)


def ellm_workspace_bytes(n_q_heads, n_kv_heads, head_dim, max_batch):
    d = _Desc()
    d.n_q_heads, d.n_kv_heads, d.head_dim, d.dtype = n_q_heads, n_kv_heads, head_dim, ELLM_BF16
    return int(lib.ellm_workspace_bytes(C.byref(d), int(max_batch)))


def ellm_pool_get_device_base(pool):
    base = C.c_void_p()
    _ret(lib.ellm_pool_get_device_base(pool, C.byref(base)), True)
    return int(base.value or 0)


def ellm_pool_get_mapping_stats(pool):
    nm, um, nu, uu = C.c_int64(), C.c_double(), C.c_int64(), C.c_double()
    _ret(lib.ellm_pool_get_mapping_stats(pool, C.byref(nm), C.byref(um), C.byref(nu), C.byref(uu)), True)
    return {"maps": nm.value, "us_map": um.value, "unmaps": nu.value, "us_unmap": uu.value}


def ellm_debug_set_table_kernels(pool, on, check=True):
    return _ret(lib.ellm_debug_set_table_kernels(pool, int(bool(on))), check)


def ellm_debug_set_async_mapping(pool, on, check=True):
    return _ret(lib.ellm_debug_set_async_mapping(pool, int(bool(on))), check)


def ellm_debug_set_copy_kernels(pool, on, check=True):
    return _ret(lib.ellm_debug_set_copy_kernels(pool, int(bool(on))), check)


def ellm_debug_fail_mapping(pool, nth, check=True):
    return _ret(lib.ellm_debug_fail_mapping(pool, int(nth)), check)


def ellm_pool_get_mapping_wait(pool):
    us = C.c_double()
    _ret(lib.ellm_pool_get_mapping_wait(pool, C.byref(us)), True)
    return us.value


def ellm_debug_fail_launch(pool, nth, check=True):
    return _ret(lib.ellm_debug_fail_launch(pool, int(nth)), check)


def ellm_pool_get_geometry(pool):
    a, b, c, d = C.c_int32(), C.c_int32(), C.c_int32(), C.c_uint64()
    _ret(lib.ellm_pool_get_geometry(pool, C.byref(a), C.byref(b), C.byref(c), C.byref(d)), True)
    return {"n_chunks": a.value, "tokens_per_chunk": b.value, "n_host_slots": c.value, "bytes_per_token": d.value}


def ellm_tensor_get_table(pool, tid):
    ns, ln = C.c_int32(), C.c_int64()
    _ret(lib.ellm_tensor_get_table(pool, tid, None, 0, C.byref(ns), C.byref(ln)), True)
    out = np.empty(ns.value, np.int32)
    _ret(lib.ellm_tensor_get_table(pool, tid, out.ctypes.data_as(_i32p), ns.value, None, None), True)
    return out, ln.value


def ellm_pool_get_owner_state(pool):
    n = ellm_pool_get_geometry(pool)["n_chunks"]
    o, s = np.empty(n, np.uint8), np.empty(n, np.uint8)
    mt, ms = np.empty(n, np.int32), np.empty(n, np.int32)
    _ret(lib.ellm_pool_get_owner_state(pool, o.ctypes.data, s.ctypes.data, mt.ctypes.data_as(_i32p),
                                       ms.ctypes.data_as(_i32p)), True)
    return o, s, mt, ms


def ellm_pool_get_host_slots(pool):
    n = ellm_pool_get_geometry(pool)["n_host_slots"]
    t, s = np.empty(max(n, 1), np.int32), np.empty(max(n, 1), np.int32)
    _ret(lib.ellm_pool_get_host_slots(pool, t.ctypes.data_as(_i32p), s.ctypes.data_as(_i32p)), True)
    return t[:n], s[:n]


def ellm_decode_plan(pool, ids, check=True):
    a, p, n = _i32(ids)
    ns = np.zeros(max(n, 1), np.int32)
    st = C.c_int32()
    rc = lib.ellm_decode_plan(pool, p, n, ns.ctypes.data_as(_i32p), C.byref(st))
    if check:
        _ret(rc, True)
        return ns[:n], st.value
    return rc


def ellm_pool_set_split_tokens(pool, split_tokens, check=True):
    return _ret(lib.ellm_pool_set_split_tokens(pool, split_tokens), check)


def ellm_pool_self_check(pool):
    return lib.ellm_pool_self_check(pool)


def ellm_pool_profile_enable(pool, max_records, check=True):
    return _ret(lib.ellm_pool_profile_enable(pool, int(max_records)), check)


def ellm_pool_profile_stride(pool, stride, check=True):
    return _ret(lib.ellm_pool_profile_stride(pool, int(stride)), check)


def ellm_pool_profile_collect(pool, cap):
    """Durations (ms) of the partial-pass kernels recorded since the last collect."""
    ms = np.zeros(max(cap, 1), np.float32)
    n = C.c_int32()
    _ret(lib.ellm_pool_profile_collect(pool, ms.ctypes.data_as(C.POINTER(C.c_float)), cap, C.byref(n)), True)
    return ms[:min(cap, n.value)]


def ellm_debug_copy(dst, src, nbytes, stream=None, check=True):
    return _ret(lib.ellm_debug_copy(_ptr(dst), _ptr(src), int(nbytes), _stream(stream)), check)


def ellm_debug_stream_read(src, nbytes, sink, stream=None, check=True):
    return _ret(lib.ellm_debug_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)), check)


def ellm_debug_kv_stream_read(pool, ids, sink, stream=None, check=True):
    _, p, n = _i32(ids)
    return _ret(lib.ellm_debug_kv_stream_read(pool, p, n, _ptr(sink), _stream(stream)), check)


def ellm_debug_set_waves(pool, percent, check=True):
    return _ret(lib.ellm_debug_set_waves(pool, int(percent)), check)
