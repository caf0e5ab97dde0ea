"""The paper's own mapping mechanism as a pool mode (Sec. 2.1.1, Sec. 3.2): chunks mapped by the
driver into each tensor's reserved address range, kernels that read the range with no table. The
parity tests of the other files run in this mode too (the `pool_mode` fixture); here: the two kinds
of kernels against each other on one pool, the driver mappings followed call by call, and what
the mode costs on the host."""
import numpy as np
import pytest
import torch

import paper_2506_15155_amd as E
import workloads as W
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def test_direct_kernels_equal_table_kernels_on_one_pool():
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=14, n_chunks=150, len_lo=64, len_hi=5000, lognormal_median=1200,
                   host_slots=24)
    st = W.draw_step(cfg, seed=83)
    B = H.Both(cfg, mode="driver")
    P = H.Both(cfg, oracle=False, mode="table")
    ids = H.load_step(B, st)
    assert H.load_step(P, st) == ids
    n_mapped = sum(len(c) for c in st.placement.chunk_ids)
    stats = E.ellm_pool_get_mapping_stats(B.pool)
    assert stats["maps"] == n_mapped and stats["unmaps"] == 0 and stats["us_map"] > 0
    assert E.ellm_pool_get_mapping_stats(P.pool) == {"maps": 0, "us_map": 0.0, "unmaps": 0, "us_unmap": 0.0}
    # fused step through the tensors' own address ranges, against the oracle and the plain pool
    rc, out, ref = B.append_decode(ids, st.k_new, st.v_new, st.q)
    assert rc == 0
    H.check_close(out, ref, "driver-mapped, direct kernels")
    rcp, outp, _ = P.append_decode(ids, st.k_new, st.v_new, st.q)
    assert rcp == 0 and torch.equal(out, outp)
    B.compare_state()
    # the same pool read through the table instead: same bits; and the appended rows are where both views agree
    E.ellm_debug_set_table_kernels(B.pool, 1)
    rc, via_table = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(via_table, out)
    E.ellm_debug_set_table_kernels(B.pool, 0)
    rc, direct = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(direct, out)
    for b in (0, 5, 13):
        for c in E.ellm_tensor_get_table(B.pool, ids[b])[0]:
            if c >= 0:
                assert np.array_equal(B.chunk_bytes_dev(int(c)), P.chunk_bytes_dev(int(c)))
    assert E.ellm_debug_set_table_kernels(P.pool, 1, check=False) == E.ERR.INVALID
    # offload takes the chunks out of the tensor's range, fetch maps other chunks there
    t = ids[5]
    n = int((E.ellm_tensor_get_table(B.pool, t)[0] >= 0).sum())
    assert B.offload(t, 0, n) == 0
    s1 = E.ellm_pool_get_mapping_stats(B.pool)
    assert s1["unmaps"] == n and s1["maps"] == n_mapped
    q = H.dev_bits(st.q)
    assert E.ellm_decode_attention(B.pool, ids, q, torch.empty_like(q), check=False) == E.ERR.NOT_RESIDENT
    _, state, _, _ = E.ellm_pool_get_owner_state(B.pool)
    free = [c for c in range(cfg.n_chunks - 1, -1, -1) if state[c] == 0][:n]
    assert B.fetch(t, 0, n, free) == 0
    s2 = E.ellm_pool_get_mapping_stats(B.pool)
    assert s2["maps"] == n_mapped + n and s2["unmaps"] == n
    rc, back = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(back, out)
    # release keeps the mapping (Sec. 2.1.2): no driver call; destroy gives everything back
    assert B.release(ids[0]) == 0
    assert E.ellm_pool_get_mapping_stats(B.pool)["unmaps"] == n
    n0 = int((E.ellm_tensor_get_table(B.pool, ids[0])[0] >= 0).sum())
    rc, t_new = B.acquire(10, cfg.max_tokens)
    assert rc == 0 and t_new == ids[0] and E.ellm_pool_get_mapping_stats(B.pool)["maps"] == n_mapped + n
    assert B.both("destroy", lambda: E.ellm_tensor_destroy(B.pool, t_new, check=False), lambda: B.orc.tensor_destroy(t_new)) == 0
    B.ids.remove(t_new)
    assert E.ellm_pool_get_mapping_stats(B.pool)["unmaps"] == n + n0
    B.compare_state()
    rc, rest = B.decode(ids[1:], st.q[1:])          # another batch, another partition: tolerance, not bits
    assert rc == 0
    H.check_close(rest, ref[1:], "after the turnover")
    print("driver calls:", E.ellm_pool_get_mapping_stats(B.pool))
    B.close()
    P.close()


def test_driver_mapped_pool_rejects_what_the_driver_cannot_map():
    # 5 kv heads of 64: a 16-token chunk is 20480 bytes ... times 1.5 = 30720, not a whole number of 4 KiB pages
    rc, _ = E.ellm_pool_create(None, None, 30720, 5, 5, 64, 2, 2, flags=E.ELLM_POOL_DRIVER_MAPPED, device_bytes=4 * 30720,
                               check=False)
    assert rc == E.ERR.INVALID and "granularity" in E.ellm_last_error()


def test_mapper_thread_orders_driver_calls_with_the_kernels():
    """The driver calls of a driver-mapped pool are made by a thread of the pool's own (Sec. 3.1: mapping
    ahead of time, unmapping off the critical path). Slots mapped ahead of their first write while
    kernels run; a compute call right behind a map call (it has to wait for the thread); chunks that leave
    one tensor while a kernel that reads them is still enqueued and at once back another tensor; the same
    sequence of calls on a second pool whose calls make their driver calls themselves: every output equals
    the oracle's within tolerance and the other pool's bit for bit, every state equals the oracle's."""
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=10, n_chunks=120, len_lo=200, len_hi=3000, lognormal_median=900)
    Tc = cfg.tokens_per_chunk
    st = W.draw_step(cfg, seed=29)
    A = H.Both(cfg, mode="driver")                       # asynchronous (the default)
    S = H.Both(cfg, oracle=False, mode="driver")         # every call waits for its own driver calls
    E.ellm_debug_set_async_mapping(S.pool, 0)
    assert E.ellm_debug_set_async_mapping(A.pool, 1) == 0
    ids = H.load_step(A, st)
    assert H.load_step(S, st) == ids
    lens = np.array([E.ellm_tensor_get_table(A.pool, t)[1] for t in ids])
    rng = np.random.default_rng(5)
    for step in range(6):
        # a few requests get the slots of their next T_c tokens mapped: nothing touches them for a while
        sub = ids[step % 3::3]
        got = E.ellm_kv_premap_ahead(A.pool, sub, Tc, 0, check=False)
        assert got == A.orc.premap_ahead(sub, Tc) and got[0] == 0
        assert E.ellm_kv_premap_ahead(S.pool, sub, Tc, 0, check=False) == got
        # append enough tokens that some requests run into the slots just mapped, decode right behind
        n_new = rng.integers(1, Tc // 3, size=cfg.batch).astype(np.int32)
        k = W.normal_bf16(rng, (int(n_new.sum()), cfg.n_kv_heads, cfg.head_dim))
        v = W.normal_bf16(rng, (int(n_new.sum()), cfg.n_kv_heads, cfg.head_dim))
        room = np.array([int((E.ellm_tensor_get_table(A.pool, t)[0] >= 0).sum()) * Tc for t in ids]) - lens
        n_new = np.minimum(n_new, np.maximum(room, 0)).astype(np.int32)
        k, v = k[:int(n_new.sum())], v[:int(n_new.sum())]
        assert A.append(ids, k, v, n_new) == 0
        assert E.ellm_kv_append(S.pool, ids, H.dev_bits(k), H.dev_bits(v), n_new, check=False) == 0
        lens += n_new
        q = W.normal_bf16(rng, (cfg.batch, cfg.n_q_heads, cfg.head_dim))
        rc, out = A.decode(ids, q)
        rcs, outs = S.decode(ids, q)
        assert rc == 0 == rcs
        rco, ref = A.orc.decode(ids, q)
        assert rco == 0
        H.check_close(out, ref, f"step {step}")
        assert torch.equal(out, outs)
        A.compare_state()
    # a decode is enqueued and not waited for; the tensors it reads are destroyed (their chunks leave the
    # ranges once the kernel is through) and new tensors take the same chunks at once
    q = W.normal_bf16(rng, (cfg.batch, cfg.n_q_heads, cfg.head_dim))
    qd = H.dev_bits(q)
    out = torch.empty_like(qd)
    assert E.ellm_decode_attention(A.pool, ids, qd, out, check=False) == 0
    rco, ref = A.orc.decode(ids, q)
    gone = ids[:4]
    for t in gone:
        assert A.both("destroy", lambda: E.ellm_tensor_destroy(A.pool, t, check=False), lambda: A.orc.tensor_destroy(t)) == 0
        A.ids.remove(t)
    fresh = []
    for i in range(4):
        t = A.create(cfg.max_tokens)
        assert A.map(t, 0, 2) == 0
        fresh.append(t)
    kk = W.normal_bf16(rng, (4 * 70, cfg.n_kv_heads, cfg.head_dim))
    vv = W.normal_bf16(rng, (4 * 70, cfg.n_kv_heads, cfg.head_dim))
    assert A.append(fresh, kk, vv, np.full(4, 70, np.int32)) == 0
    torch.cuda.synchronize()
    H.check_close(out, ref, "decode enqueued before its tensors were destroyed")
    q2 = W.normal_bf16(rng, (4, cfg.n_q_heads, cfg.head_dim))
    rc, out2 = A.decode(fresh, q2)
    rco, ref2 = A.orc.decode(fresh, q2)
    assert rc == 0 == rco
    H.check_close(out2, ref2, "tensors backed by chunks that had just left other ranges")
    A.compare_state()
    assert E.ellm_pool_sync(A.pool, check=False) == 0
    sa, ss = E.ellm_pool_get_mapping_stats(A.pool), E.ellm_pool_get_mapping_stats(S.pool)
    assert sa["unmaps"] > 0 and sa["maps"] > ss["maps"] > 0
    print("mapper thread:", sa, "callers waited", round(E.ellm_pool_get_mapping_wait(A.pool), 1), "us; inline:", ss,
          "waited", round(E.ellm_pool_get_mapping_wait(S.pool), 1), "us")
    A.close()
    S.close()


def test_a_refused_mapping_stops_the_pool_before_any_launch():
    """The mapper thread meets a driver error (forced by the test hook: the mapping is simply not made):
    the next call that would launch a kernel on the pool returns ELLM_ERR_HIP and launches nothing, so no
    kernel ever reads the slot that has no chunk behind it; the host state is untouched by the failed
    calls; the pool can still be destroyed."""
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=4, n_chunks=40, len_lo=100, len_hi=900, lognormal_median=400)
    st = W.draw_step(cfg, seed=31)
    B = H.Both(cfg, oracle=False, mode="driver")
    ids = H.load_step(B, st)
    rc, out0 = B.decode(ids, st.q)
    assert rc == 0
    E.ellm_debug_fail_mapping(B.pool, 2)
    assert E.ellm_kv_premap_ahead(B.pool, ids, cfg.tokens_per_chunk, 0) >= 2      # the second mapping asked for is refused
    assert E.ellm_pool_sync(B.pool, check=False) == E.ERR.HIP                     # the thread has got there
    q = H.dev_bits(st.q)
    out = torch.zeros_like(q)
    rc = E.ellm_decode_attention(B.pool, ids, q, out, check=False)
    assert rc == E.ERR.HIP and "refused" in E.ellm_last_error()
    torch.cuda.synchronize()
    assert not out.any()                                                          # nothing ran
    lens = [E.ellm_tensor_get_table(B.pool, t)[1] for t in ids]
    k, v = H.dev_bits(st.k_new), H.dev_bits(st.v_new)
    assert E.ellm_kv_append(B.pool, ids, k, v, check=False) == E.ERR.HIP
    assert E.ellm_kv_append_decode(B.pool, ids, k, v, q, out, check=False) == E.ERR.HIP
    assert [E.ellm_tensor_get_table(B.pool, t)[1] for t in ids] == lens           # no length moved
    assert E.ellm_pool_sync(B.pool, check=False) == E.ERR.HIP
    assert E.ellm_debug_fail_mapping(B.pool, -1, check=False) == E.ERR.INVALID
    B.close()
