"""ctypes front end of the C oracle (ellm_oracle.c). TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

MODE_CHUNKED, MODE_TWIN, MODE_ONLINE = 0, 1, 2

_i32p = C.POINTER(C.c_int32)
_u8p = C.POINTER(C.c_uint8)
_u16p = C.POINTER(C.c_uint16)
_f64p = C.POINTER(C.c_double)


class OracleError(Exception):
    def __init__(self, code: int, what: str):
        super().__init__(f"oracle {what}: code {code}")
        self.code = code


def load(path: str | None = None) -> C.CDLL:
    path = path or _build.build(force=False)
    lib = C.CDLL(path)
    lib.orc_pool_create.restype = C.c_void_p
    lib.orc_pool_create.argtypes = [C.c_int32, C.c_uint32, C.c_int32, C.c_int, C.c_int, C.c_int,
                                    C.c_int32, C.c_int32, _u8p, C.c_int]
    lib.orc_pool_destroy.argtypes = [C.c_void_p]
    lib.orc_pool_destroy.restype = None
    lib.orc_tokens_per_chunk.argtypes = [C.c_void_p]
    lib.orc_tensor_create.argtypes = [C.c_void_p, C.c_int64, _i32p]
    lib.orc_tensor_destroy.argtypes = [C.c_void_p, C.c_int32]
    lib.orc_tensor_release.argtypes = [C.c_void_p, C.c_int32]
    lib.orc_tensor_acquire.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_uint32, _i32p]
    lib.orc_tensor_is_released.argtypes = [C.c_void_p, C.c_int32]
    lib.orc_kv_premap_next.argtypes = [C.c_void_p, _i32p, C.c_int32, C.c_uint32, _i32p]
    lib.orc_kv_premap_ahead.argtypes = [C.c_void_p, _i32p, C.c_int32, C.c_int64, C.c_uint32, _i32p]
    lib.orc_pool_set_logical_host_slots.argtypes = [C.c_void_p, C.c_int32]
    lib.orc_pool_get_logical_host_slots.argtypes = [C.c_void_p]
    lib.orc_pool_slo_configure.argtypes = [C.c_void_p, C.c_double, C.c_double, C.c_double, C.c_int32, C.c_int32]
    lib.orc_pool_slo_observe.argtypes = [C.c_void_p, C.c_double, C.c_double, _i32p]
    lib.orc_tensor_map_chunks.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _i32p, C.c_uint32]
    lib.orc_tensor_unmap_chunks.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
    lib.orc_pool_transfer.argtypes = [C.c_void_p, _i32p, C.c_int32, C.c_int]
    lib.orc_pool_set_act_busy.argtypes = [C.c_void_p, _i32p, C.c_int32, C.c_int]
    lib.orc_kv_append.argtypes = [C.c_void_p, _i32p, C.c_int32, _i32p, _u16p, _u16p]
    lib.orc_chunk_offload.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
    lib.orc_chunk_fetch.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _i32p]
    lib.orc_tensor_get_table.argtypes = [C.c_void_p, C.c_int32, _i32p, C.c_int32, _i32p, C.POINTER(C.c_int64)]
    lib.orc_pool_get_owner_state.argtypes = [C.c_void_p, _u8p, _u8p, _i32p, _i32p]
    lib.orc_pool_get_owner_state.restype = None
    lib.orc_pool_get_host_slots.argtypes = [C.c_void_p, _i32p, _i32p]
    lib.orc_pool_get_host_slots.restype = None
    lib.orc_chunk_set_bytes.argtypes = [C.c_void_p, C.c_int32, _u8p]
    lib.orc_chunk_get_bytes.argtypes = [C.c_void_p, C.c_int32, _u8p]
    lib.orc_host_slot_get_bytes.argtypes = [C.c_void_p, C.c_int32, _u8p]
    lib.orc_check_invariants.argtypes = [C.c_void_p]
    lib.orc_decode_attention.argtypes = [C.c_void_p, _i32p, C.c_int32, _u16p, C.c_double, C.c_int, C.c_int, _f64p]
    lib.orc_attention_weights.argtypes = [C.c_void_p, C.c_int32, _u16p, C.c_int, C.c_double, _f64p]
    return lib


def _i32(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(_i32p)


def _u16(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.uint16)
    return arr, arr.ctypes.data_as(_u16p)


class OraclePool:
    """The oracle's own pool + tensors + byte image. Methods return the C return code for the
    state-changing calls (so tests can compare error codes with the GPU library's) and raise only
    on misuse of the wrapper itself."""

    def __init__(self, n_chunks, chunk_bytes, n_host, Hq, Hkv, D, max_tensors, max_slots,
                 initial_owner=None, keep_twin=True, lib=None):
        self.lib = lib or load()
        own = None
        if initial_owner is not None:
            self._own = np.ascontiguousarray(initial_owner, dtype=np.uint8)
            assert self._own.size == n_chunks
            own = self._own.ctypes.data_as(_u8p)
        self.h = self.lib.orc_pool_create(n_chunks, chunk_bytes, n_host, Hq, Hkv, D, max_tensors,
                                          max_slots, own, int(keep_twin))
        if not self.h:
            raise OracleError(-1, "pool_create")
        self.n_chunks, self.chunk_bytes, self.n_host = n_chunks, chunk_bytes, n_host
        self.Hq, self.Hkv, self.D = Hq, Hkv, D
        self.tokens_per_chunk = self.lib.orc_tokens_per_chunk(self.h)

    def close(self):
        if self.h:
            self.lib.orc_pool_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- state machine (return codes) ----
    def tensor_create(self, max_tokens):
        out = C.c_int32(-1)
        rc = self.lib.orc_tensor_create(self.h, int(max_tokens), C.byref(out))
        return rc, out.value

    def tensor_destroy(self, tid):
        return self.lib.orc_tensor_destroy(self.h, tid)

    def release(self, tid):
        return self.lib.orc_tensor_release(self.h, tid)

    def acquire(self, need_tokens, max_tokens, flags=0):
        out = C.c_int32(-1)
        rc = self.lib.orc_tensor_acquire(self.h, int(need_tokens), int(max_tokens), int(flags), C.byref(out))
        return rc, out.value

    def is_released(self, tid):
        return self.lib.orc_tensor_is_released(self.h, tid)

    def premap_next(self, ids, flags=0):
        a, p = _i32(ids)
        out = C.c_int32(0)
        rc = self.lib.orc_kv_premap_next(self.h, p, a.size, int(flags), C.byref(out))
        return rc, out.value

    def premap_ahead(self, ids, tokens_ahead, flags=0):
        a, p = _i32(ids)
        out = C.c_int32(0)
        rc = self.lib.orc_kv_premap_ahead(self.h, p, a.size, int(tokens_ahead), int(flags), C.byref(out))
        return rc, out.value

    def set_logical_host_slots(self, n):
        return self.lib.orc_pool_set_logical_host_slots(self.h, int(n))

    def logical_host_slots(self):
        return self.lib.orc_pool_get_logical_host_slots(self.h)

    def slo_configure(self, ttft_slo, tpot_slo, alpha=2.0, window=5, threshold=3):
        return self.lib.orc_pool_slo_configure(self.h, float(ttft_slo), float(tpot_slo), float(alpha), int(window),
                                               int(threshold))

    def slo_observe(self, ttft, tpot):
        out = C.c_int32(0)
        rc = self.lib.orc_pool_slo_observe(self.h, float(ttft), float(tpot), C.byref(out))
        return rc, out.value

    def map_chunks(self, tid, first, n, chunk_ids=None, flags=0):
        _, p = _i32(chunk_ids)
        return self.lib.orc_tensor_map_chunks(self.h, tid, first, n, p, flags)

    def unmap_chunks(self, tid, first, n):
        return self.lib.orc_tensor_unmap_chunks(self.h, tid, first, n)

    def transfer(self, chunk_ids, new_owner):
        a, p = _i32(chunk_ids)
        return self.lib.orc_pool_transfer(self.h, p, a.size, new_owner)

    def set_act_busy(self, chunk_ids, busy):
        a, p = _i32(chunk_ids)
        return self.lib.orc_pool_set_act_busy(self.h, p, a.size, int(busy))

    def append(self, ids, k_new, v_new, n_new=None):
        a, p = _i32(ids)
        _, pn = _i32(n_new)
        _, pk = _u16(k_new)
        _, pv = _u16(v_new)
        return self.lib.orc_kv_append(self.h, p, a.size, pn, pk, pv)

    def offload(self, tid, first, n):
        return self.lib.orc_chunk_offload(self.h, tid, first, n)

    def fetch(self, tid, first, n, chunk_ids=None):
        _, p = _i32(chunk_ids)
        return self.lib.orc_chunk_fetch(self.h, tid, first, n, p)

    # ---- read-out ----
    def table(self, tid):
        ns, ln = C.c_int32(0), C.c_int64(0)
        rc = self.lib.orc_tensor_get_table(self.h, tid, None, 0, C.byref(ns), C.byref(ln))
        if rc:
            raise OracleError(rc, "get_table")
        out = np.empty(ns.value, dtype=np.int32)
        self.lib.orc_tensor_get_table(self.h, tid, out.ctypes.data_as(_i32p), ns.value, None, None)
        return out, ln.value

    def owner_state(self):
        o = np.empty(self.n_chunks, np.uint8)
        s = np.empty(self.n_chunks, np.uint8)
        mt = np.empty(self.n_chunks, np.int32)
        ms = np.empty(self.n_chunks, np.int32)
        self.lib.orc_pool_get_owner_state(self.h, o.ctypes.data_as(_u8p), s.ctypes.data_as(_u8p),
                                          mt.ctypes.data_as(_i32p), ms.ctypes.data_as(_i32p))
        return o, s, mt, ms

    def host_slots(self):
        t = np.empty(max(self.n_host, 1), np.int32)
        s = np.empty(max(self.n_host, 1), np.int32)
        self.lib.orc_pool_get_host_slots(self.h, t.ctypes.data_as(_i32p), s.ctypes.data_as(_i32p))
        return t[:self.n_host], s[:self.n_host]

    def chunk_set_bytes(self, c, data):
        a = np.ascontiguousarray(data, dtype=np.uint8)
        assert a.size == self.chunk_bytes
        return self.lib.orc_chunk_set_bytes(self.h, c, a.ctypes.data_as(_u8p))

    def chunk_bytes_of(self, c):
        out = np.empty(self.chunk_bytes, np.uint8)
        rc = self.lib.orc_chunk_get_bytes(self.h, c, out.ctypes.data_as(_u8p))
        if rc:
            raise OracleError(rc, "chunk_get_bytes")
        return out

    def host_slot_bytes(self, s):
        out = np.empty(self.chunk_bytes, np.uint8)
        rc = self.lib.orc_host_slot_get_bytes(self.h, s, out.ctypes.data_as(_u8p))
        if rc:
            raise OracleError(rc, "host_slot_get_bytes")
        return out

    def check_invariants(self):
        return self.lib.orc_check_invariants(self.h)

    # ---- attention ----
    def decode(self, ids, q, scale=0.0, mode=MODE_CHUNKED, threads=None):
        """fp64 attention output [batch][Hq][D]; returns (rc, out)."""
        a, p = _i32(ids)
        qa, pq = _u16(q)
        out = np.zeros((a.size, self.Hq, self.D), dtype=np.float64)
        threads = threads or os.cpu_count() or 1
        rc = self.lib.orc_decode_attention(self.h, p, a.size, pq, float(scale), mode, int(threads),
                                           out.ctypes.data_as(_f64p))
        return rc, out

    def weights(self, tid, q_head_vec, h, scale=0.0):
        _, ln = self.table(tid)
        qa, pq = _u16(q_head_vec)
        w = np.zeros(ln, dtype=np.float64)
        rc = self.lib.orc_attention_weights(self.h, tid, pq, h, float(scale), w.ctypes.data_as(_f64p))
        if rc:
            raise OracleError(rc, "weights")
        return w
