"""GPU parity at the full sizes of the configurations, in the launch configuration bench.py times
(automatic cut into per-wave shares): every output where the oracle finishes in seconds, otherwise sampled
requests the oracle computes one by one, plus the elastic ten-step twin run."""
import numpy as np
import pytest
import torch

import paper_2506_15155_amd as E
import workloads as W
from oracle.model import OraclePool
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def test_llama8b_full_every_output(pool_mode):
    """The 8B-shaped configuration at its full size: all 64 requests, every output element."""
    cfg = W.CONFIGS["llama8b"]
    st = W.draw_step(cfg)
    B = H.Both(cfg)
    ids = H.load_step(B, st)
    assert B.append(ids, st.k_new, st.v_new) == 0
    rc, out = B.decode(ids, st.q)
    rco, ref = B.orc.decode(ids, st.q)
    assert rc == 0 and rco == 0
    mx, mean = H.check_close(out, ref, "llama8b full")
    print(f"llama8b full: {int(st.lens.sum())} tokens, max-abs {mx:.2e} mean-abs {mean:.2e}")
    B.compare_state()
    rc, again = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(out, again)
    B.close()


def bits_np(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run_sampled(cfg, n_sample):
    """History drawn on the device (seeded) and written through the library for every request; the
    same values go to the oracle for a seeded sample of requests (always with the longest and the
    shortest one, spread evenly over the length order), which it then computes one by one."""
    st = W.draw_step(cfg, with_values=False)
    owner = st.placement.owner if cfg.act_fraction > 0 else None
    dev = torch.empty(cfg.n_chunks * cfg.chunk_bytes, dtype=torch.uint8, device="cuda")
    dev.view(torch.int16).fill_(H.POISON)
    pool = E.ellm_pool_create(dev, None, cfg.chunk_bytes, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                              cfg.batch, cfg.max_slots, owner)
    orc = OraclePool(cfg.n_chunks, cfg.chunk_bytes, 0, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                     cfg.batch, cfg.max_slots, owner, False)
    if len(st.placement.act_busy):
        assert E.ellm_pool_set_act_busy(pool, st.placement.act_busy, 1, check=False) == 0
        assert orc.set_act_busy(st.placement.act_busy, 1) == 0
    # requests at evenly spaced ranks of the length order: the shortest, the longest and, from 11
    # samples on, at least one from every length decile
    order = np.argsort(st.lens, kind="stable")
    ranks = np.unique(np.rint(np.linspace(0, cfg.batch - 1, min(n_sample, cfg.batch))).astype(int))
    sample = sorted(int(order[r]) for r in ranks)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed)
    shape = (cfg.n_kv_heads, cfg.head_dim)
    ids = []
    for b in range(cfg.batch):
        rc, tid = E.ellm_tensor_create(pool, cfg.max_tokens, check=False)
        assert (rc, tid) == orc.tensor_create(cfg.max_tokens) and rc == 0
        cid = st.placement.chunk_ids[b]
        assert E.ellm_tensor_map_chunks(pool, tid, 0, len(cid), cid, check=False) == 0
        assert orc.map_chunks(tid, 0, len(cid), cid) == 0
        ids.append(tid)
        n = int(st.lens[b]) - 1
        k = torch.randn((n,) + shape, generator=gen, device="cuda").to(torch.bfloat16)
        v = torch.randn((n,) + shape, generator=gen, device="cuda").to(torch.bfloat16)
        assert E.ellm_kv_append(pool, [tid], k, v, [n], check=False) == 0
        if b in sample:
            assert orc.append([tid], bits_np(k), bits_np(v), [n]) == 0
        torch.cuda.synchronize()
        del k, v
    k1 = torch.randn((cfg.batch,) + shape, generator=gen, device="cuda").to(torch.bfloat16)
    v1 = torch.randn((cfg.batch,) + shape, generator=gen, device="cuda").to(torch.bfloat16)
    q = torch.randn((cfg.batch, cfg.n_q_heads, cfg.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    out = torch.empty_like(q)
    assert E.ellm_kv_append(pool, ids, k1, v1, check=False) == 0
    assert E.ellm_decode_attention(pool, ids, q, out, check=False) == 0
    torch.cuda.synchronize()
    sid = [ids[b] for b in sample]
    assert orc.append(sid, bits_np(k1)[sample], bits_np(v1)[sample]) == 0
    rco, ref = orc.decode(sid, bits_np(q)[sample])
    assert rco == 0
    mx, mean = H.check_close(out[sample], ref, cfg.name)
    print(f"{cfg.name} full size: {int(st.lens.sum())} tokens in {cfg.batch} requests, sampled {sample} "
          f"(lengths {[int(st.lens[b]) for b in sample]}): max-abs {mx:.2e} mean-abs {mean:.2e}")
    # properties that hold at any size: finite everywhere, bounded by the largest |V| (a convex
    # combination), same bits on a second run
    got = H.out_f64(out)
    assert np.isfinite(got).all() and np.abs(got).max() < 8.0
    out2 = torch.empty_like(out)
    assert E.ellm_decode_attention(pool, ids, q, out2, check=False) == 0
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    # tables of every request, lengths of the sampled ones, owner/state arrays: bit-exact
    for a, b_ in zip(E.ellm_pool_get_owner_state(pool), orc.owner_state()):
        assert np.array_equal(a, b_)
    for b in range(cfg.batch):
        ta, la = E.ellm_tensor_get_table(pool, ids[b])
        tb, lb = orc.table(ids[b])
        assert np.array_equal(ta, tb) and la == int(st.lens[b])
        assert lb == (la if b in sample else 0)
    assert E.ellm_pool_self_check(pool) == 0 and orc.check_invariants() == 0
    # the sampled requests' chunk bytes (appended rows, poison elsewhere untouched by the library)
    for b in sample[:2]:
        c = int(st.placement.chunk_ids[b][-1])
        used = 2 * cfg.n_kv_heads * cfg.tokens_per_chunk * cfg.head_dim * 2
        d = dev[c * cfg.chunk_bytes:(c + 1) * cfg.chunk_bytes].cpu().numpy()
        o = orc.chunk_bytes_of(c)
        rows = int(st.lens[b]) - (len(st.placement.chunk_ids[b]) - 1) * cfg.tokens_per_chunk
        dd = d[:used].reshape(cfg.n_kv_heads * 2, cfg.tokens_per_chunk, cfg.head_dim * 2)
        oo = o[:used].reshape(cfg.n_kv_heads * 2, cfg.tokens_per_chunk, cfg.head_dim * 2)
        assert np.array_equal(dd[:, :rows], oo[:, :rows])
        assert (dd[:, rows:].view(np.uint16) == H.POISON).all()      # rows past the length were never written
    torch.cuda.synchronize()
    E.ellm_pool_destroy(pool)
    orc.close()


def test_mha13b_full_sampled():
    """13B-shaped MHA layer at full size (128 requests, 2k..16k tokens, 102-token chunks, half the
    pool busy activations): 16 requests, at least one from every length decile, against the oracle."""
    run_sampled(W.CONFIGS["mha13b"], 16)


def test_long70b_full_every_request():
    """70B-shaped long-context layer at full size (16 requests of 32k..128k tokens, group of 8):
    every request against the oracle."""
    run_sampled(W.CONFIGS["long70b"], 16)


def test_elastic_ten_steps_twin_run(pool_mode):
    """Ten decode steps with the pool reshaped before each: 30 % of the activation region handed
    to the KV side, all chunks of 25 % of the requests offloaded to pinned host and fetched back
    into whatever chunks the pool picks, then map-ahead, append and decode. A twin pool takes the
    same appends with no remapping: the two outputs must agree bit for bit, the remapped pool's
    state must match the oracle's bit for bit, its output the oracle's within tolerance."""
    cfg = W.CONFIGS["elastic"]
    st = W.draw_step(cfg)
    A = H.Both(cfg, owner=st.placement.owner)
    T = H.Both(cfg, owner=st.placement.owner, oracle=False, mode="table")     # the twin is always a plain pool
    ids = H.load_step(A, st)
    idt = H.load_step(T, st)
    assert ids == idt
    rng = np.random.default_rng(cfg.seed + 4)
    lens = st.lens.copy() - 1                  # before the first step's append
    tc = cfg.tokens_per_chunk
    shape = (cfg.batch, cfg.n_kv_heads, cfg.head_dim)
    moved = 0
    for step in range(10):
        # deflate the activation side: 30 % of what it still owns goes idle and changes owner
        owner, state, _, _ = E.ellm_pool_get_owner_state(A.pool)
        act = np.flatnonzero(owner == E.ELLM_OWNER_ACT).astype(np.int32)
        give = np.sort(rng.choice(act, size=int(0.3 * len(act)), replace=False)).astype(np.int32)
        if len(give):
            busy = give[state[give] == E.ELLM_CHUNK_BUSY]
            if len(busy):
                assert A.both("idle", lambda: E.ellm_pool_set_act_busy(A.pool, busy, 0, check=False),
                              lambda: A.orc.set_act_busy(busy, 0)) == 0
            assert A.both("transfer", lambda: E.ellm_pool_transfer(A.pool, give, E.ELLM_OWNER_KV, check=False),
                          lambda: A.orc.transfer(give, E.ELLM_OWNER_KV)) == 0
        # offload a quarter of the requests, then bring them back
        sel = np.sort(rng.choice(cfg.batch, size=cfg.batch // 4, replace=False))
        before = {}
        for b in sel:
            n_slots = -(-int(lens[b]) // tc)
            before[int(b)] = E.ellm_tensor_get_table(A.pool, ids[b])[0][:n_slots].copy()
            assert A.offload(ids[b], 0, n_slots) == 0
        A.compare_state()
        for b in sel:
            n_slots = -(-int(lens[b]) // tc)
            assert A.fetch(ids[b], 0, n_slots) == 0
            after = E.ellm_tensor_get_table(A.pool, ids[b])[0][:n_slots]
            moved += int((after != before[int(b)]).sum())
        E.ellm_pool_sync(A.pool)
        # map ahead, append, decode on both pools
        for b in np.flatnonzero(lens % tc == 0):
            s = int(lens[b]) // tc
            if E.ellm_tensor_get_table(A.pool, ids[b])[0][s] != -1:
                continue                       # the initial placement already covers the first new token
            assert A.map(ids[b], s, 1, None, E.ELLM_MAP_ALLOW_INFLATE) == 0
            assert T.map(idt[b], s, 1, None, E.ELLM_MAP_ALLOW_INFLATE) == 0
        k1, v1, q = W.normal_bf16(rng, shape), W.normal_bf16(rng, shape), \
            W.normal_bf16(rng, (cfg.batch, cfg.n_q_heads, cfg.head_dim))
        assert A.append(ids, k1, v1) == 0 and T.append(idt, k1, v1) == 0
        lens += 1
        rc, out = A.decode(ids, q)
        rct, twin = T.decode(idt, q)
        rco, ref = A.orc.decode(ids, q)
        assert rc == 0 and rct == 0 and rco == 0
        assert torch.equal(out, twin), f"step {step}: remapped and unremapped pools disagree"
        H.check_close(out, ref, f"elastic step {step}")
        A.compare_state()
    assert moved > 0, "the round trips never changed a chunk id: not a remap test"
    # migrated bytes: every written row of the chunks of the last offloaded request equals the
    # oracle's image (the oracle's unwritten rows are zero, the device's are poison)
    b = int(sel[-1])
    n_slots = -(-int(lens[b]) // tc)
    for s_, c in enumerate(E.ellm_tensor_get_table(A.pool, ids[b])[0][:n_slots]):
        rows = min(tc, int(lens[b]) - s_ * tc)
        used = 2 * cfg.n_kv_heads * tc * cfg.head_dim * 2
        dd = A.chunk_bytes_dev(int(c))[:used].reshape(cfg.n_kv_heads * 2, tc, cfg.head_dim * 2)
        oo = A.orc.chunk_bytes_of(int(c))[:used].reshape(cfg.n_kv_heads * 2, tc, cfg.head_dim * 2)
        assert np.array_equal(dd[:, :rows], oo[:, :rows])
    print(f"elastic: 10 steps, {moved} slot remaps through the host")
    A.close()
    T.close()
