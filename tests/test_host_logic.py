"""Host state machine of the library (pool, chunk tables, error paths) against the oracle's own
pool model, through the C ABI on a pool created with ELLM_POOL_METADATA_ONLY (no device needed).
Tables, owner/state arrays, host-slot maps and return codes must agree bit for bit after every call
of seeded random call sequences. The two sides share no code: the library is C++ (pool_core.cpp),
the oracle plain C (ellm_oracle.c)."""
import re
import os

import numpy as np
import pytest

import paper_2506_15155_amd as E
from oracle.model import OraclePool

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DUMMY = 4096   # non-NULL stand-in for device pointers; never dereferenced in metadata-only mode


class Pair:
    """The library pool and the oracle pool driven by the same calls."""

    def __init__(self, n_chunks=48, n_host=10, Hq=8, Hkv=8, D=64, Tc=16, max_tensors=6, max_slots=12, owner=None):
        cb = Tc * 2 * Hkv * D * 2
        self.lib = E.ellm_pool_create(None, None, cb, Hq, Hkv, D, max_tensors, max_slots, owner,
                                      flags=E.ELLM_POOL_METADATA_ONLY, device_bytes=n_chunks * cb,
                                      host_bytes=n_host * cb)
        self.orc = OraclePool(n_chunks, cb, n_host, Hq, Hkv, D, max_tensors, max_slots, owner, keep_twin=False)
        self.n_chunks, self.n_host, self.Tc, self.max_tensors = n_chunks, n_host, Tc, max_tensors
        self.Hkv, self.D = Hkv, D

    def close(self):
        E.ellm_pool_destroy(self.lib)
        self.orc.close()

    def compare(self):
        lo, ls, lmt, lms = E.ellm_pool_get_owner_state(self.lib)
        oo, os_, omt, oms = self.orc.owner_state()
        assert np.array_equal(lo, oo) and np.array_equal(ls, os_)
        assert np.array_equal(lmt, omt) and np.array_equal(lms, oms)
        assert E.ellm_pool_get_logical_host_slots(self.lib) == self.orc.logical_host_slots()
        lt, lsl = E.ellm_pool_get_host_slots(self.lib)
        ot, osl = self.orc.host_slots()
        assert np.array_equal(lt, ot) and np.array_equal(lsl, osl)
        for tid in range(self.max_tensors):
            try:
                tab, ln = E.ellm_tensor_get_table(self.lib, tid)
                alive = True
            except E.EllmError:
                alive = False
            try:
                otab, oln = self.orc.table(tid)
                oalive = True
            except Exception:
                oalive = False
            assert alive == oalive
            if alive:
                assert np.array_equal(tab, otab) and ln == oln
                assert E.ellm_tensor_is_released(self.lib, tid) == self.orc.is_released(tid)
        assert E.ellm_pool_self_check(self.lib) == 0
        assert self.orc.check_invariants() == 0
        # no physical chunk backs two slots
        mapped = [int(e) for tid in range(self.max_tensors) if self._alive(tid)
                  for e in E.ellm_tensor_get_table(self.lib, tid)[0] if e >= 0]
        assert len(mapped) == len(set(mapped))

    def _alive(self, tid):
        try:
            E.ellm_tensor_get_table(self.lib, tid)
            return True
        except E.EllmError:
            return False


def random_walk(seed, steps=600, **kw):
    rng = np.random.default_rng(seed)
    owner = (rng.random(kw.get("n_chunks", 48)) < 0.35).astype(np.uint8)
    P = Pair(owner=owner, **kw)
    if seed % 2:
        assert E.ellm_pool_slo_configure(P.lib, 100.0, 5.0, 2.0, 5, 3, check=False) == 0 == P.orc.slo_configure(100.0, 5.0)
    seen_codes = set()
    for _ in range(steps):
        op = rng.choice(["create", "destroy", "map", "map_ids", "unmap", "transfer", "busy", "append",
                         "decode", "offload", "fetch", "fetch_ids", "release", "acquire", "premap", "logical", "slo"],
                        p=[.07, .03, .13, .07, .03, .07, .07, .17, .05, .07, .05, .03, .05, .04, .03, .01, .03])
        alive = [t for t in range(P.max_tensors) if P._alive(t)]
        if alive and rng.random() < 0.8:
            # mostly plausible arguments, so the walk reaches deep states (full host buffer, long tensors)
            tid = int(rng.choice(alive))
            tab, ln = E.ellm_tensor_get_table(P.lib, tid)
            first = int(rng.integers(0, tab.size))
            n = int(rng.integers(0, min(5, tab.size - first) + 1))
        else:
            tid = int(rng.integers(-1, P.max_tensors + 1))
            first = int(rng.integers(-1, 13))
            n = int(rng.integers(-1, 6))
        ids = rng.integers(-1, P.n_chunks + 1, size=max(n, 0)).astype(np.int32)
        if op == "create":
            mt = int(rng.integers(0, 16 * 13))
            a = E.ellm_tensor_create(P.lib, mt, check=False)
            b = P.orc.tensor_create(mt)
            assert a == b, (op, a, b)
            rc = a[0]
        elif op == "destroy":
            rc = E.ellm_tensor_destroy(P.lib, tid, check=False)
            assert rc == P.orc.tensor_destroy(tid)
        elif op == "map":
            fl = int(rng.integers(0, 2))
            rc = E.ellm_tensor_map_chunks(P.lib, tid, first, n, None, fl, check=False)
            assert rc == P.orc.map_chunks(tid, first, n, None, fl), op
        elif op == "map_ids":
            fl = int(rng.integers(0, 2))
            rc = E.ellm_tensor_map_chunks(P.lib, tid, first, n, ids if n > 0 else None, fl, check=False)
            assert rc == P.orc.map_chunks(tid, first, n, ids if n > 0 else None, fl), op
        elif op == "unmap":
            rc = E.ellm_tensor_unmap_chunks(P.lib, tid, first, n, check=False)
            assert rc == P.orc.unmap_chunks(tid, first, n), op
        elif op == "transfer":
            own = int(rng.integers(0, 3))
            rc = E.ellm_pool_transfer(P.lib, ids, own, check=False)
            assert rc == P.orc.transfer(ids, own), op
        elif op == "busy":
            busy = int(rng.integers(0, 2))
            rc = E.ellm_pool_set_act_busy(P.lib, ids, busy, check=False)
            assert rc == P.orc.set_act_busy(ids, busy), op
        elif op == "append":
            nb = int(rng.integers(0, 4))
            tids = rng.integers(-1, P.max_tensors, size=nb).astype(np.int32)
            if alive and rng.random() < 0.8:
                tids = rng.choice(alive, size=min(nb, len(alive)), replace=False).astype(np.int32)
                nb = tids.size
            nn = rng.integers(-1, 40, size=nb).astype(np.int32)
            tot = int(np.clip(nn, 0, None).sum())
            kv = np.zeros((max(tot, 1), P.Hkv, P.D), np.uint16)
            use_n = None if (nb and rng.random() < 0.3) else nn
            rc = E.ellm_kv_append(P.lib, tids, DUMMY, DUMMY, use_n, stream=0, check=False)
            kv1 = np.zeros((max(nb, 1), P.Hkv, P.D), np.uint16)
            assert rc == P.orc.append(tids, kv if use_n is not None else kv1, kv if use_n is not None else kv1, use_n), op
        elif op == "decode":
            nb = int(rng.integers(0, 4))
            tids = rng.integers(-1, P.max_tensors, size=nb).astype(np.int32)
            rc = E.ellm_decode_attention(P.lib, tids, DUMMY, DUMMY, stream=0, check=False)
            orc_rc, _ = P.orc.decode(tids, np.zeros((max(nb, 1), 8, P.D), np.uint16), threads=1)
            # with no device behind it the library validates, then reports NO_DEVICE instead of OK
            assert (rc == orc_rc) or (orc_rc == 0 and rc == (E.ERR.NO_DEVICE if nb else 0)), (rc, orc_rc)
        elif op == "release":
            rc = E.ellm_tensor_release(P.lib, tid, check=False)
            assert rc == P.orc.release(tid), op
        elif op == "acquire":
            need = int(rng.integers(-1, 16 * 8))
            mt = int(rng.integers(0, 16 * 13))
            fl = int(rng.integers(0, 2))
            a = E.ellm_tensor_acquire(P.lib, need, mt, fl, check=False)
            b = P.orc.acquire(need, mt, fl)
            assert a[0] == b[0] and (a[0] != 0 or a[1] == b[1]), (op, a, b)
            rc = a[0]
        elif op == "premap":
            nb = int(rng.integers(0, 4))
            tids = rng.integers(-1, P.max_tensors, size=nb).astype(np.int32)
            if alive and rng.random() < 0.8:
                tids = rng.choice(alive, size=min(nb, len(alive)), replace=False).astype(np.int32)
            fl = int(rng.integers(0, 2))
            if rng.random() < 0.5:
                a = E.ellm_kv_premap_next(P.lib, tids, fl, check=False)
                b = P.orc.premap_next(tids, fl)
            else:
                ahead = int(rng.integers(0, 40))
                a = E.ellm_kv_premap_ahead(P.lib, tids, ahead, fl, check=False)
                b = P.orc.premap_ahead(tids, ahead, fl)
            assert a[0] == b[0] and (a[0] != 0 or a[1] == b[1]), (op, a, b)
            rc = a[0]
        elif op == "logical":
            n_l = int(rng.integers(-1, P.n_host + 2))
            rc = E.ellm_pool_set_logical_host_slots(P.lib, n_l, check=False)
            assert rc == P.orc.set_logical_host_slots(n_l), op
        elif op == "slo":
            lat = (float(rng.choice([-1.0, 10.0, 200.0])), float(rng.choice([-1.0, 1.0, 9.0])))
            a = E.ellm_pool_slo_observe(P.lib, *lat, check=False)
            assert a == P.orc.slo_observe(*lat), (op, a)
            rc = a[0]
        elif op == "offload":
            rc = E.ellm_chunk_deflate_to_host(P.lib, tid, first, n, check=False)
            assert rc == P.orc.offload(tid, first, n), op
        elif op == "fetch":
            rc = E.ellm_chunk_inflate_from_host(P.lib, tid, first, n, None, check=False)
            assert rc == P.orc.fetch(tid, first, n, None), op
        else:
            rc = E.ellm_chunk_inflate_from_host(P.lib, tid, first, n, ids if n > 0 else None, check=False)
            assert rc == P.orc.fetch(tid, first, n, ids if n > 0 else None), op
        seen_codes.add(rc)
        P.compare()
    P.close()
    return seen_codes


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_random_call_sequences_match_oracle(seed):
    random_walk(seed)


def test_random_walks_reach_every_error_code():
    seen = set()
    for seed in range(10, 18):
        seen |= random_walk(seed, steps=600, n_host=2 if seed % 2 else 10)
    for code in (E.ERR.OK, E.ERR.INVALID, E.ERR.OOM, E.ERR.OWNED, E.ERR.UNMAPPED, E.ERR.NOT_RESIDENT,
                 E.ERR.RANGE, E.ERR.EMPTY, E.ERR.HOST_FULL):
        assert code in seen, code


def test_non_power_of_two_tokens_per_chunk():
    """13B-shaped geometry: 2 MiB chunks, bpt 20480 -> 102 tokens per chunk, 8192 bytes of slack."""
    P = E.ellm_pool_create(None, None, 2 << 20, 40, 40, 128, 2, 162, flags=1, device_bytes=8 * (2 << 20))
    g = E.ellm_pool_get_geometry(P)
    assert g["tokens_per_chunk"] == 102 and g["bytes_per_token"] == 20480 and g["n_chunks"] == 8
    t = E.ellm_tensor_create(P, 16384 + 102)
    tab, ln = E.ellm_tensor_get_table(P, t)
    assert tab.size == 162 and ln == 0
    assert E.ellm_tensor_create(P, 102 * 162 + 1, check=False)[0] == E.ERR.RANGE
    E.ellm_pool_destroy(P)


def test_failed_calls_change_nothing():
    P = Pair()
    t = E.ellm_tensor_create(P.lib, 64)
    P.orc.tensor_create(64)
    before = E.ellm_pool_get_owner_state(P.lib)
    assert E.ellm_tensor_map_chunks(P.lib, t, 0, 3, [5, 6, 5], check=False) == E.ERR.OWNED      # repeated id
    assert E.ellm_tensor_map_chunks(P.lib, t, 0, 3, [5, 6, 99], check=False) == E.ERR.RANGE
    assert E.ellm_tensor_map_chunks(P.lib, t, 2, 3, None, check=False) == E.ERR.RANGE
    assert E.ellm_kv_append(P.lib, [t], DUMMY, DUMMY, stream=0, check=False) == E.ERR.UNMAPPED
    assert E.ellm_decode_attention(P.lib, [t], DUMMY, DUMMY, stream=0, check=False) == E.ERR.EMPTY
    assert "no token" in E.ellm_last_error()
    after = E.ellm_pool_get_owner_state(P.lib)
    for a, b in zip(before, after):
        assert np.array_equal(a, b)
    assert (E.ellm_tensor_get_table(P.lib, t)[0] == -1).all()
    P.close()


def test_fused_append_decode_checks_on_host():
    """The fused call validates like an append of one token each, then like a decode over the
    lengths after it; when it fails, or has no device to run on, nothing has changed. Each code is
    the one the oracle's pool gives for append-then-decode on the same state."""
    P = Pair(n_chunks=8, n_host=2, max_tensors=3, max_slots=2)
    t = E.ellm_tensor_create(P.lib, 32)
    u = E.ellm_tensor_create(P.lib, 16)
    P.orc.tensor_create(32)
    P.orc.tensor_create(16)

    def fused(ids, k=DUMMY, q=DUMMY):
        return E.ellm_kv_append_decode(P.lib, ids, k, k, q, DUMMY, stream=0, check=False)

    one = np.zeros((1, P.Hkv, P.D), np.uint16)
    assert fused([t]) == E.ERR.UNMAPPED == P.orc.append([t], one, one)
    assert E.ellm_tensor_map_chunks(P.lib, t, 0, 1, None, check=False) == 0 == P.orc.map_chunks(t, 0, 1, None, 0)
    assert fused([t, u]) == E.ERR.UNMAPPED                 # the second request has no chunk
    assert fused([t, t]) == E.ERR.INVALID
    assert fused([t], k=None) == E.ERR.INVALID
    assert fused([t], q=None) == E.ERR.INVALID
    assert fused([7]) == E.ERR.INVALID
    assert fused([]) == 0                                   # empty batch: nothing to do
    assert fused([t]) == E.ERR.NO_DEVICE                    # all checks passed; no device to run on
    assert E.ellm_tensor_get_table(P.lib, t)[1] == 0        # and the length was not advanced
    # a slot below the new token that is on the host: the decode half of the checks catches it
    assert E.ellm_tensor_map_chunks(P.lib, t, 1, 1, None, check=False) == 0 == P.orc.map_chunks(t, 1, 1, None, 0)
    toks = np.zeros((16, P.Hkv, P.D), np.uint16)
    assert E.ellm_kv_append(P.lib, [t], DUMMY, DUMMY, [16], stream=0, check=False) == 0 == P.orc.append([t], toks, toks, [16])
    assert E.ellm_chunk_deflate_to_host(P.lib, t, 0, 1, check=False) == 0 == P.orc.offload(t, 0, 1)
    assert fused([t]) == E.ERR.NOT_RESIDENT
    assert P.orc.append([t], one, one) == 0 and P.orc.decode([t], np.zeros((1, 8, P.D), np.uint16))[0] == E.ERR.NOT_RESIDENT
    assert E.ellm_tensor_get_table(P.lib, t)[1] == 16
    # range: a tensor that is full
    assert E.ellm_tensor_map_chunks(P.lib, u, 0, 1, None, check=False) == 0
    assert E.ellm_kv_append(P.lib, [u], DUMMY, DUMMY, [16], stream=0, check=False) == 0
    assert fused([u]) == E.ERR.RANGE
    P.close()


def test_pool_create_rejects_bad_geometry():
    ok = dict(device_buf=None, host_buf=None, chunk_bytes=32768, n_q_heads=8, n_kv_heads=8, head_dim=64,
              max_tensors=4, max_slots_per_tensor=4, flags=1, device_bytes=4 * 32768)
    assert E.ellm_pool_create(**ok, check=False)[0] == 0
    for k, v in [("head_dim", 96), ("n_kv_heads", 3), ("chunk_bytes", 1000), ("chunk_bytes", 1024),
                 ("device_bytes", 100), ("max_tensors", 0), ("flags", 3)]:
        bad = dict(ok)
        bad[k] = v
        assert E.ellm_pool_create(**bad, check=False)[0] == E.ERR.INVALID, k
    # a real (non metadata-only) pool needs a device pointer
    bad = dict(ok)
    bad["flags"] = 0
    assert E.ellm_pool_create(**bad, check=False)[0] == E.ERR.INVALID
    # a driver-mapped pool brings its own memory, and is never metadata-only (checked before any device call)
    bad = dict(ok)
    bad["flags"] = E.ELLM_POOL_DRIVER_MAPPED | E.ELLM_POOL_METADATA_ONLY
    assert E.ellm_pool_create(**bad, check=False)[0] == E.ERR.INVALID
    bad = dict(ok)
    bad["flags"], bad["device_buf"] = E.ELLM_POOL_DRIVER_MAPPED, DUMMY
    assert E.ellm_pool_create(**bad, check=False)[0] == E.ERR.INVALID


def test_driver_mapped_buffer_rejects_bad_arguments_before_any_device_call():
    assert E.ellm_debug_vmm_buffer_create(0, 4, check=False)[0] == E.ERR.INVALID
    assert E.ellm_debug_vmm_buffer_create(2 << 20, 0, check=False)[0] == E.ERR.INVALID
    assert E.ellm_debug_vmm_buffer_destroy(4096, check=False) == E.ERR.INVALID


def test_library_exports_every_declared_symbol():
    """Every function include/ellm.h declares is exported by the built library and bound in Python."""
    text = open(os.path.join(ROOT, "include", "ellm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ellm_[a-z_0-9]+)\s*\(", text))
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(E.lib, name), name
        assert callable(getattr(E, name)), name
    assert declared == set(E.binding.EXPORTED)


def test_split_plan_depends_only_on_lengths():
    """The sequence partition is a function of the batch's lengths and the geometry, not of which
    physical chunks back the tensors."""
    plans = []
    for perm_seed in (0, 1):
        rng = np.random.default_rng(perm_seed)
        cb = 2 << 20
        P = E.ellm_pool_create(None, None, cb, 32, 8, 128, 8, 17, flags=1, device_bytes=256 * cb)
        perm = list(rng.permutation(256))
        ids = []
        for L in (64, 700, 3000, 8192):
            t = E.ellm_tensor_create(P, 8704)
            ns = -(-L // 512)
            E.ellm_tensor_map_chunks(P, t, 0, ns, [perm.pop() for _ in range(ns)])
            E.ellm_kv_append(P, [t], DUMMY, DUMMY, [L], stream=0)
            ids.append(t)
        ns, S = E.ellm_decode_plan(P, ids)
        plans.append((list(ns), S))
        # tiles are dealt out evenly to at most 1024 / 8 waves per kv head (one per SIMD; the figure assumed
        # without a device); a wave holds at most S / 64 of them, and each request boundary adds at most one partial
        tiles = [-(-L // 64) for L in (64, 700, 3000, 8192)]
        assert S > 0 and S % 64 == 0 and S // 64 == -(-sum(tiles) // 128)
        assert all(n >= -(-t // (S // 64)) for n, t in zip(ns, tiles))
        assert sum(ns) <= 128 + len(tiles) - 1
        E.ellm_pool_set_split_tokens(P, 64)
        ns1, S1 = E.ellm_decode_plan(P, ids)
        assert S1 == 64 and list(ns1) == tiles
        E.ellm_pool_destroy(P)
    assert plans[0] == plans[1]


def test_workspace_bytes_bounds_every_plan():
    """ellm_workspace_bytes is an upper bound of what any launch's partition needs: checked against the
    partition the library itself reports for the five workload shapes at their seeded lengths, for a
    batch of many short requests (most request boundaries per wave), one of 300 requests (three
    launches) and a single long request."""
    import workloads as W
    cases = [(W.CONFIGS[n], None) for n in ("tiny", "llama8b", "mha13b", "elastic", "long70b")]
    cases.append((W.scaled(W.CONFIGS["llama8b"], batch=128), np.full(128, 65)))
    cases.append((W.scaled(W.CONFIGS["llama8b"], batch=300), None))
    cases.append((W.scaled(W.CONFIGS["long70b"], batch=1), np.array([131072])))
    for cfg, lens in cases:
        if lens is None:
            lens = W.draw_lengths(cfg, np.random.default_rng(cfg.seed))
        Tc, B = cfg.tokens_per_chunk, cfg.batch
        need = [int(-(-int(l) // Tc)) for l in lens]
        P = E.ellm_pool_create(None, None, cfg.chunk_bytes, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, B, max(need),
                               flags=1, device_bytes=(sum(need) + 1) * cfg.chunk_bytes)
        ids = []
        for b in range(B):
            t = E.ellm_tensor_create(P, need[b] * Tc)
            E.ellm_tensor_map_chunks(P, t, 0, need[b])
            ids.append(t)
        E.ellm_kv_append(P, ids, DUMMY, DUMMY, np.asarray(lens, np.int32), stream=0)
        n_split, _ = E.ellm_decode_plan(P, ids)
        slot_bytes = cfg.group * (cfg.head_dim + 2) * 4
        cap = E.ellm_workspace_bytes(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, B)
        assert cap > 0 and cap % slot_bytes == 0
        assert cap == (1024 + cfg.n_kv_heads * (min(B, 128) - 1)) * slot_bytes       # no device here: 1024 SIMDs assumed
        for b0 in range(0, B, 128):                                                   # one launch per 128 requests
            ns = n_split[b0:b0 + 128]
            slots = cfg.n_kv_heads * int(ns[ns > 1].sum())
            assert slots * slot_bytes <= cap, (cfg.name, B, slots)
        E.ellm_pool_destroy(P)
    assert E.ellm_workspace_bytes(32, 8, 96, 4) == 0 and E.ellm_workspace_bytes(32, 8, 128, 0) == 0


def test_refused_launch_leaves_whole_groups():
    """An append of more than 128 requests works in launches of 128. When the runtime refuses one (forced
    here by the test hook), the groups before it are appended completely and the rest not at all: the
    state equals the oracle's after an append of exactly those groups."""
    Pn = Pair(n_chunks=320, n_host=0, max_tensors=300, max_slots=2)
    ids = []
    for i in range(300):
        t = E.ellm_tensor_create(Pn.lib, 32)
        assert Pn.orc.tensor_create(32) == (0, t)
        assert E.ellm_tensor_map_chunks(Pn.lib, t, 0, 1, None, check=False) == 0 == Pn.orc.map_chunks(t, 0, 1, None, 0)
        ids.append(t)
    n_new = (np.arange(300) % 5 + 1).astype(np.int32)
    E.ellm_debug_fail_launch(Pn.lib, 2)
    rc = E.ellm_kv_append(Pn.lib, ids, DUMMY, DUMMY, n_new, stream=0, check=False)
    assert rc == E.ERR.HIP and "refused" in E.ellm_last_error()
    rows = np.zeros((int(n_new[:128].sum()), Pn.Hkv, Pn.D), np.uint16)
    assert Pn.orc.append(ids[:128], rows, rows, n_new[:128]) == 0
    Pn.compare()
    lens = [E.ellm_tensor_get_table(Pn.lib, t)[1] for t in ids]
    assert lens[:128] == list(n_new[:128]) and not any(lens[128:])
    # the hook is spent: the rest goes through, and a check that fails still changes nothing
    assert E.ellm_kv_append(Pn.lib, ids[128:], DUMMY, DUMMY, n_new[128:], stream=0, check=False) == 0
    assert E.ellm_kv_append(Pn.lib, ids, DUMMY, DUMMY, np.full(300, 32, np.int32), stream=0, check=False) == E.ERR.RANGE
    assert [E.ellm_tensor_get_table(Pn.lib, t)[1] for t in ids] == list(n_new)
    Pn.close()


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU measurement: asking for more exits with a message, before any GPU work."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""

