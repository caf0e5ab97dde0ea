"""GPU tests of the rules around the kernels: the logical host buffer driven through real offloads,
chunks handed to the activation side while their offload copy is still queued, calls on two streams,
a refused launch in the middle of a call that works in several launches, and the workspace bound."""
import numpy as np
import pytest
import torch

import paper_2506_15155_amd as E
import workloads as W
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def test_logical_host_buffer_on_device():
    """Sec. 2.3.2 on a device pool: offloads fill the logical part of the host buffer; shrinking it
    below what is parked refuses further offloads but leaves every parked byte in pinned memory;
    growing it again (by time-to-first-token violations) admits offloads again. State and return
    codes against the oracle after every call, parked bytes by memcmp, attention output after the
    chunks have come back into other places."""
    cfg = W.scaled(W.CONFIGS["tiny"], batch=4, host_slots=12)
    st = W.draw_step(cfg, seed=25)        # slots per request: 9, 3, 14, 1
    B = H.Both(cfg)
    poison = np.full(cfg.chunk_bytes // 2, H.POISON, np.uint16).view(np.uint8)
    for c in range(cfg.n_chunks):
        B.orc.chunk_set_bytes(c, poison)
    ids = H.load_step(B, st)
    assert B.append(ids, st.k_new, st.v_new) == 0
    rc, before = B.decode(ids, st.q)
    assert rc == 0
    slots = [int(-(-int(l) // cfg.tokens_per_chunk)) for l in st.lens]
    order = np.argsort(slots)                       # two requests that fit the buffer together, a third that must not
    a, b, c = int(order[0]), int(order[1]), int(order[2])
    assert slots[a] + slots[b] <= 11

    def both(name, lib_call, orc_call):
        r = B.both(name, lib_call, orc_call)
        B.compare_state()
        return r

    def observe(ttft, tpot):
        got = E.ellm_pool_slo_observe(B.pool, ttft, tpot, check=False)
        assert got == B.orc.slo_observe(ttft, tpot)
        assert E.ellm_pool_get_logical_host_slots(B.pool) == B.orc.logical_host_slots() == got[1]
        B.compare_state()
        return got[1]

    assert both("slo", lambda: E.ellm_pool_slo_configure(B.pool, 100.0, 10.0, 2.0, 5, 3, check=False),
                lambda: B.orc.slo_configure(100.0, 10.0, 2.0, 5, 3)) == 0
    parked = {}                                     # host slot -> bytes of the chunk parked there
    for r in (a, b):
        tab, _ = E.ellm_tensor_get_table(B.pool, ids[r])
        pre = [B.chunk_bytes_dev(int(x)) for x in tab[:slots[r]]]
        assert B.offload(ids[r], 0, slots[r]) == 0
        B.compare_state()
        tabh, _ = E.ellm_tensor_get_table(B.pool, ids[r])
        for i in range(slots[r]):
            parked[-int(tabh[i]) - 2] = pre[i]
    E.ellm_pool_sync(B.pool)
    n_parked = slots[a] + slots[b]
    # time-per-output-token violations: 12 -> 6 -> 3 -> 1, below what is parked
    size = 12
    while size > 1:
        for _ in range(3):
            size = observe(-1.0, 50.0)
    assert size == 1 < n_parked
    assert B.offload(ids[c], 0, 1) == E.ERR.HOST_FULL
    B.compare_state()
    th, _ = E.ellm_pool_get_host_slots(B.pool)
    assert int((th >= 0).sum()) == n_parked          # nothing was evicted
    for hs, want in parked.items():                  # and every parked byte is where it was
        assert np.array_equal(B.host_slot_bytes(hs), want)
        assert np.array_equal(B.orc.host_slot_bytes(hs), want)
    # the parked requests cannot decode; the resident ones can, bits unchanged
    q = H.dev_bits(st.q)
    assert E.ellm_decode_attention(B.pool, ids, q, torch.empty_like(q), check=False) == E.ERR.NOT_RESIDENT
    keep = [r for r in range(cfg.batch) if r not in (a, b)]
    rc, part = B.decode([ids[r] for r in keep], st.q[keep])
    assert rc == 0 and torch.equal(part, before[keep])
    # time-to-first-token violations grow it: 1 -> 2 -> 4 -> 8 -> 12 (capacity)
    sizes = []
    while size < 12:
        for _ in range(3):
            size = observe(500.0, -1.0)
        sizes.append(size)
        # an offload is admitted as soon as the logical size exceeds what is parked
        want = 0 if size >= n_parked + 1 else E.ERR.HOST_FULL
        assert B.offload(ids[c], 0, 1) == want
        B.compare_state()
        if want == 0:
            assert B.fetch(ids[c], 0, 1) == 0
            E.ellm_pool_sync(B.pool)
    assert sizes[-1] == 12 and sizes[:3] == [2, 4, 8]
    # bring everything back, into the highest free chunks (other places than before)
    for r in (a, b):
        _, s, _, _ = E.ellm_pool_get_owner_state(B.pool)
        free = [x for x in range(cfg.n_chunks - 1, -1, -1) if s[x] == 0][:slots[r]]
        assert B.fetch(ids[r], 0, slots[r], free) == 0
        B.compare_state()
    E.ellm_pool_sync(B.pool)
    rc, after = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(before, after)
    rco, ref = B.orc.decode(ids, st.q)
    assert rco == 0
    H.check_close(after, ref, "after the logical-buffer round trip")
    B.close()


def test_offloaded_chunks_handed_to_the_activation_side():
    """The elastic flow of Sec. 2.2.2: KV chunks are offloaded to make room for activations. The
    offload frees the device chunks while their copies are still queued; handing them to the
    activation side (and marking them busy) must not return before the copies have read them, since
    whoever fills them next runs on streams the library does not see. Here another stream overwrites
    them at once; the parked bytes must still be the KV bytes, and the request must decode as before
    after coming back."""
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=3, n_chunks=48, len_lo=2000, len_hi=6000, lognormal_median=4000,
                   host_slots=40)
    st = W.draw_step(cfg, seed=29)
    B = H.Both(cfg)
    ids = H.load_step(B, st)
    assert B.append(ids, st.k_new, st.v_new) == 0
    rc, before = B.decode(ids, st.q)
    assert rc == 0
    other = torch.cuda.Stream()
    cb = cfg.chunk_bytes
    for r in range(cfg.batch):
        tab, _ = E.ellm_tensor_get_table(B.pool, ids[r])
        live = [int(x) for x in tab if x >= 0]
        pre = [B.chunk_bytes_dev(x) for x in live]
        torch.cuda.synchronize()
        assert B.offload(ids[r], 0, len(live)) == 0                       # 2 MiB copies, queued
        give = np.array(live, np.int32)
        assert B.both("to act", lambda: E.ellm_pool_transfer(B.pool, give, E.ELLM_OWNER_ACT, check=False),
                      lambda: B.orc.transfer(give, E.ELLM_OWNER_ACT)) == 0
        assert B.both("busy", lambda: E.ellm_pool_set_act_busy(B.pool, give, 1, check=False),
                      lambda: B.orc.set_act_busy(give, 1)) == 0
        with torch.cuda.stream(other):                                     # "activations" land in the chunks
            for x in live:
                B.dev[x * cb:(x + 1) * cb].fill_(0xAB)
        B.compare_state()
        tabh, _ = E.ellm_tensor_get_table(B.pool, ids[r])
        E.ellm_pool_sync(B.pool)
        other.synchronize()
        for i in range(len(live)):
            assert np.array_equal(B.host_slot_bytes(-int(tabh[i]) - 2), pre[i]), (r, i)
        # the activations are done: chunks idle, back to the KV side, and the request comes home
        assert B.both("idle", lambda: E.ellm_pool_set_act_busy(B.pool, give, 0, check=False),
                      lambda: B.orc.set_act_busy(give, 0)) == 0
        assert B.both("to kv", lambda: E.ellm_pool_transfer(B.pool, give, E.ELLM_OWNER_KV, check=False),
                      lambda: B.orc.transfer(give, E.ELLM_OWNER_KV)) == 0
        assert B.fetch(ids[r], 0, len(live), give[::-1].copy()) == 0        # same chunks, other order
        B.compare_state()
    rc, after = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(before, after)
    B.close()


def test_calls_on_two_streams_are_ordered():
    """The append / decode calls of a pool form one sequence whatever streams they are given: a
    decode on another stream than the append before it waits for that append (and for the table
    changes pushed with it) without any synchronisation by the caller."""
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=10, n_chunks=160, len_lo=500, len_hi=5000, lognormal_median=2500)
    st = W.draw_step(cfg, seed=37)
    B = H.Both(cfg, max_tensors=cfg.batch + 1)
    ids = H.load_step(B, st)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    kd, vd, qd = H.dev_bits(st.k_new), H.dev_bits(st.v_new), H.dev_bits(st.q)
    out = torch.empty_like(qd)
    torch.cuda.synchronize()
    # a long multi-token append keeps s1 busy; then the one-token append on s1 and the decode on s2
    tail = B.create(cfg.max_tokens)
    assert B.map(tail, 0, 16) == 0
    big = torch.zeros((8000, cfg.n_kv_heads, cfg.head_dim), dtype=torch.int16, device="cuda")
    assert E.ellm_kv_append(B.pool, [tail], big, big, [8000], stream=s1, check=False) == 0
    assert E.ellm_kv_append(B.pool, ids, kd, vd, stream=s1, check=False) == 0
    assert E.ellm_decode_attention(B.pool, ids, qd, out, stream=s2, check=False) == 0
    s2.synchronize()
    assert B.orc.append([tail], np.zeros((8000, cfg.n_kv_heads, cfg.head_dim), np.uint16),
                        np.zeros((8000, cfg.n_kv_heads, cfg.head_dim), np.uint16), [8000]) == 0
    assert B.orc.append(ids, st.k_new, st.v_new) == 0
    rco, ref = B.orc.decode(ids, st.q)
    assert rco == 0
    H.check_close(out, ref, "decode on a second stream")
    torch.cuda.synchronize()
    B.compare_state()
    B.close()


def test_refused_launch_in_a_fused_call_leaves_whole_groups():
    """300 requests are three launches. The second is refused (test hook: nothing is launched, as when
    the runtime returns an error): the first 128 requests have been appended and decoded, rows,
    lengths and output, the other 172 are untouched."""
    cfg = W.Config("wide", 8, 300, 8, 2, 64, 16 * (2 * 2 * 64 * 2), 700, 32, "uniform", 1, 31)
    st = W.draw_step(cfg, seed=5)
    B = H.Both(cfg)
    ids = H.load_step(B, st)
    kd, vd, qd = H.dev_bits(st.k_new), H.dev_bits(st.v_new), H.dev_bits(st.q)
    out = torch.full_like(qd, 123)
    E.ellm_debug_fail_launch(B.pool, 2)
    rc = E.ellm_kv_append_decode(B.pool, ids, kd, vd, qd, out, check=False)
    torch.cuda.synchronize()
    assert rc == E.ERR.HIP and "refused" in E.ellm_last_error()
    assert B.orc.append(ids[:128], st.k_new[:128], st.v_new[:128]) == 0
    B.compare_state()
    rco, ref = B.orc.decode(ids[:128], st.q[:128])
    assert rco == 0
    H.check_close(out[:128], ref, "requests of the accepted launch")
    assert (out[128:] == 123).all()
    # the rest goes through afterwards
    rc, out2, ref2 = B.append_decode(ids[128:], st.k_new[128:], st.v_new[128:], st.q[128:])
    assert rc == 0
    H.check_close(out2, ref2, "the remaining requests")
    B.compare_state()
    B.close()


def test_workspace_bound_on_the_device():
    """ellm_workspace_bytes, evaluated for the GPU the test runs on, bounds what the partitions of the
    library's own plans need, and a prepared pool decodes without allocating anything further."""
    simds = torch.cuda.get_device_properties(0).multi_processor_count * 4
    for name in ("llama8b", "long70b"):
        cfg = W.scaled(W.CONFIGS[name], batch=8, n_chunks=2100 if name == "long70b" else 200)
        slot_bytes = cfg.group * (cfg.head_dim + 2) * 4
        cap = E.ellm_workspace_bytes(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.batch)
        assert cap == (simds + cfg.n_kv_heads * (cfg.batch - 1)) * slot_bytes
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=8, n_chunks=200)
    st = W.draw_step(cfg, seed=3)
    B = H.Both(cfg)
    E.ellm_pool_prepare(B.pool)
    ids = H.load_step(B, st)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    rc, out, ref = B.append_decode(ids, st.k_new, st.v_new, st.q)
    assert rc == 0
    H.check_close(out, ref, "prepared pool")
    n_split, _ = E.ellm_decode_plan(B.pool, ids)
    assert cfg.n_kv_heads * int(n_split[n_split > 1].sum()) * cfg.group * (cfg.head_dim + 2) * 4 <= \
        E.ellm_workspace_bytes(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.batch)
    B.close()
    del free0


@pytest.mark.parametrize("seed", [11, 12])
def test_random_walk_of_every_call_on_the_gpu(pool_mode, seed):
    """A seeded walk of a few hundred calls of every kind, valid and invalid ones mixed, through the
    library on the GPU and the oracle side by side: every return code equal; tables, owners, states and
    host-slot maps equal after every tenth call; every decode that both sides accept within tolerance;
    at the end every chunk and every host slot byte for byte."""
    # 8 q / 2 kv heads of 128, 16-token chunks of 16 KiB, 8 tensor handles of at most 8 slots
    cfg = W.Config("walk", 9, 8, 8, 2, 128, 16 * (2 * 2 * 128 * 2), 56, 16 * 8, "uniform", 1, 128, host_slots=12)
    Tc, Hkv, Hq, D = cfg.tokens_per_chunk, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim
    rng = np.random.default_rng(seed)
    owner = (rng.random(cfg.n_chunks) < 0.25).astype(np.uint8)
    B = H.Both(cfg, owner=owner, keep_twin=True, max_tensors=8)
    poison = np.full(cfg.chunk_bytes // 2, H.POISON, np.uint16).view(np.uint8)
    for c in range(cfg.n_chunks):
        B.orc.chunk_set_bytes(c, poison)
    P, O = B.pool, B.orc
    n_ok = n_dec = 0
    if seed == 12:
        E.ellm_debug_set_copy_kernels(P, 1)      # offload / fetch through the library's copy kernel in this one

    def some_ids(k=None):
        k = int(rng.integers(1, 5)) if k is None else k
        if rng.random() < 0.85:
            live = [t for t in range(8) if O.is_released(t) == 0]
            if live:
                return list(rng.choice(live, size=min(k, len(live)), replace=False).astype(np.int32))
        return list(rng.integers(-1, 9, size=k).astype(np.int32))

    for it in range(320):
        op = rng.choice(["create", "destroy", "map", "unmap", "append", "fused", "decode", "offload", "fetch", "release",
                         "acquire", "premap", "transfer", "busy", "logical"],
                        p=[.08, .03, .12, .03, .16, .12, .12, .07, .07, .03, .04, .05, .04, .02, .02])
        rc = None
        if op == "create":
            mt = int(rng.integers(1, 8 * Tc + 1))
            a, b = E.ellm_tensor_create(P, mt, check=False), O.tensor_create(mt)
            assert a[0] == b[0] and (a[0] != 0 or a[1] == b[1]), (op, a, b)
            rc = a[0]
            if rc == 0 and a[1] not in B.ids:
                B.ids.append(a[1])
        elif op == "destroy":
            t = int(some_ids(1)[0])
            rc = E.ellm_tensor_destroy(P, t, check=False)
            assert rc == O.tensor_destroy(t), op
            if rc == 0:
                B.ids.remove(t)
        elif op == "map":
            t, first, n, fl = int(some_ids(1)[0]), int(rng.integers(0, 8)), int(rng.integers(1, 4)), int(rng.integers(0, 2))
            cids = None if rng.random() < 0.7 else rng.integers(0, cfg.n_chunks, size=n).astype(np.int32)
            rc = B.map(t, first, n, cids, fl)
        elif op == "unmap":
            t, first, n = int(some_ids(1)[0]), int(rng.integers(0, 8)), int(rng.integers(1, 3))
            rc = B.both(op, lambda: E.ellm_tensor_unmap_chunks(P, t, first, n, check=False), lambda: O.unmap_chunks(t, first, n))
        elif op == "append":
            ids = some_ids()
            n_new = rng.integers(0, 2 * Tc, size=len(ids)).astype(np.int32)
            k = W.normal_bf16(rng, (int(n_new.sum()), Hkv, D))
            v = W.normal_bf16(rng, (int(n_new.sum()), Hkv, D))
            rc = B.append(ids, k, v, n_new)
        elif op == "fused":
            ids = some_ids()
            k, v = W.normal_bf16(rng, (len(ids), Hkv, D)), W.normal_bf16(rng, (len(ids), Hkv, D))
            q = W.normal_bf16(rng, (len(ids), Hq, D))
            # accepted: the oracle must accept the append and then the decode; refused: nothing may have
            # changed (the comparison of the states that follows sees to that)
            rc, out, ref = B.append_decode(ids, k, v, q)
            if rc == 0:
                H.check_close(out, ref, f"call {it} fused")
                n_dec += 1
        elif op == "decode":
            ids = some_ids()
            q = W.normal_bf16(rng, (len(ids), Hq, D))
            rc, out = B.decode(ids, q)
            rco, ref = O.decode(ids, q)
            assert rc == rco, (op, rc, rco, E.ellm_last_error())
            if rc == 0:
                H.check_close(out, ref, f"call {it} decode")
                n_dec += 1
        elif op == "offload":
            t, first, n = int(some_ids(1)[0]), int(rng.integers(0, 6)), int(rng.integers(1, 4))
            rc = B.offload(t, first, n)
        elif op == "fetch":
            t, first, n = int(some_ids(1)[0]), int(rng.integers(0, 6)), int(rng.integers(1, 4))
            rc = B.fetch(t, first, n)
        elif op == "release":
            t = int(some_ids(1)[0])
            rc = B.both(op, lambda: E.ellm_tensor_release(P, t, check=False), lambda: O.release(t))
        elif op == "acquire":
            rc, _ = B.acquire(int(rng.integers(0, 6 * Tc)), int(rng.integers(1, 8 * Tc + 1)), int(rng.integers(0, 2)))
        elif op == "premap":
            ids, fl = some_ids(), int(rng.integers(0, 2))
            if rng.random() < 0.5:
                a, b = E.ellm_kv_premap_next(P, ids, fl, check=False), O.premap_next(ids, fl)
            else:
                ahead = int(rng.integers(0, 3 * Tc))
                a, b = E.ellm_kv_premap_ahead(P, ids, ahead, fl, check=False), O.premap_ahead(ids, ahead, fl)
            assert a[0] == b[0] and (a[0] != 0 or a[1] == b[1]), (op, a, b)
            rc = a[0]
        elif op == "transfer":
            cids = rng.integers(0, cfg.n_chunks, size=int(rng.integers(1, 5))).astype(np.int32)
            to = int(rng.integers(0, 2))
            rc = B.both(op, lambda: E.ellm_pool_transfer(P, cids, to, check=False), lambda: O.transfer(cids, to))
        elif op == "busy":
            cids = rng.integers(0, cfg.n_chunks, size=int(rng.integers(1, 4))).astype(np.int32)
            busy = int(rng.integers(0, 2))
            rc = B.both(op, lambda: E.ellm_pool_set_act_busy(P, cids, busy, check=False), lambda: O.set_act_busy(cids, busy))
        else:
            n_l = int(rng.integers(-1, cfg.host_slots + 2))
            rc = B.both(op, lambda: E.ellm_pool_set_logical_host_slots(P, n_l, check=False),
                        lambda: O.set_logical_host_slots(n_l))
        n_ok += rc == 0
        if it % 10 == 9 or (op == "fused" and rc != 0):
            B.compare_state()
    B.compare_state()
    assert E.ellm_pool_sync(P, check=False) == 0
    torch.cuda.synchronize()
    owner_now, state_now, _, _ = E.ellm_pool_get_owner_state(P)
    for c in range(cfg.n_chunks):
        # chunks that belong to busy activations are the caller's to write; all others must match
        assert np.array_equal(B.chunk_bytes_dev(c), O.chunk_bytes_of(c)), c
    slot_tensor, _ = E.ellm_pool_get_host_slots(P)
    for s in range(cfg.host_slots):
        if slot_tensor[s] >= 0:
            assert np.array_equal(B.host_slot_bytes(s), O.host_slot_bytes(s)), s
    del owner_now, state_now
    assert n_ok >= 80 and n_dec >= 10, (n_ok, n_dec)
    print(f"walk seed {seed} ({pool_mode}): {n_ok} of 320 calls accepted, {n_dec} decodes compared")
    B.close()
