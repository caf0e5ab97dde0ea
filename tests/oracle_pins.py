"""Pins for the CPU oracle: each function checks the oracle against something the mathematics or
a library fixes, and raises AssertionError when the oracle is wrong. They take the loaded oracle
library as an argument so that deliberately broken builds of the oracle can be run through the
same checks (see test_oracle_mutants.py)."""
from __future__ import annotations

import math

import numpy as np

import workloads as W
from oracle.model import OraclePool, MODE_CHUNKED, MODE_TWIN, MODE_ONLINE


def f64(bits):
    return W.f32_from_bf16_bits(bits).astype(np.float64)


def make_pool(lib, Hq=8, Hkv=8, D=64, Tc=16, n_chunks=64, n_host=8, max_tensors=8, max_slots=32, owner=None):
    chunk_bytes = Tc * 2 * Hkv * D * 2
    return OraclePool(n_chunks, chunk_bytes, n_host, Hq, Hkv, D, max_tensors, max_slots, owner, True, lib)


def fill(pool, lens, rng, chunk_perm=None, k=None, v=None):
    """Create one tensor per length, map shuffled chunks, append everything. Returns ids, K, V lists."""
    Tc = pool.tokens_per_chunk
    perm = list(chunk_perm if chunk_perm is not None else rng.permutation(pool.n_chunks))
    ids, Ks, Vs = [], [], []
    for i, L in enumerate(lens):
        rc, tid = pool.tensor_create(max(L, 1))
        assert rc == 0
        ns = -(-L // Tc)
        cid = [perm.pop() for _ in range(ns)]
        assert pool.map_chunks(tid, 0, ns, cid) == 0
        Kb = k[i] if k is not None else W.normal_bf16(rng, (L, pool.Hkv, pool.D))
        Vb = v[i] if v is not None else W.normal_bf16(rng, (L, pool.Hkv, pool.D))
        assert pool.append([tid], Kb, Vb, [L]) == 0
        ids.append(tid); Ks.append(Kb); Vs.append(Vb)
    return ids, Ks, Vs


# ---------------------------------------------------------------------------------------------
def pin_sdpa_library(lib):
    """Special case that reduces to a library routine: torch's scaled_dot_product_attention on CPU
    in fp64 with the kv heads repeated G times (contiguous groups). MHA, GQA-4 and GQA-8."""
    import torch
    import torch.nn.functional as F
    for (Hq, Hkv, D, Tc, lens, seed) in [(8, 8, 64, 16, [16, 33, 256, 1], 1), (8, 2, 128, 7, [5, 50, 23], 2),
                                         (16, 2, 128, 12, [40, 13], 3)]:
        rng = np.random.default_rng(seed)
        pool = make_pool(lib, Hq, Hkv, D, Tc, n_chunks=96, max_slots=64)
        ids, Ks, Vs = fill(pool, lens, rng)
        q = W.normal_bf16(rng, (len(lens), Hq, D))
        rc, out = pool.decode(ids, q)
        assert rc == 0
        G = Hq // Hkv
        for b, L in enumerate(lens):
            qt = torch.from_numpy(f64(q[b]))[:, None, :]                               # [Hq,1,D]
            kt = torch.from_numpy(f64(Ks[b])).permute(1, 0, 2).repeat_interleave(G, 0)  # [Hq,L,D]
            vt = torch.from_numpy(f64(Vs[b])).permute(1, 0, 2).repeat_interleave(G, 0)
            ref = F.scaled_dot_product_attention(qt, kt, vt)[:, 0, :].numpy()
            assert np.abs(out[b] - ref).max() <= 1e-12, (Hq, Hkv, b, np.abs(out[b] - ref).max())
        pool.close()


def pin_single_token(lib):
    """L = 1: the only weight is 1, so the output is V[0] exactly."""
    rng = np.random.default_rng(4)
    pool = make_pool(lib, 8, 4, 64, 16)
    ids, Ks, Vs = fill(pool, [1], rng)
    q = W.normal_bf16(rng, (1, 8, 64))
    rc, out = pool.decode(ids, q)
    assert rc == 0
    for h in range(8):
        assert np.array_equal(out[0, h], f64(Vs[0][0, h // 2]))
    pool.close()


def pin_zero_query_is_mean(lib):
    """q = 0: all scores equal, so the output is the arithmetic mean of V over the tokens."""
    rng = np.random.default_rng(5)
    pool = make_pool(lib, 8, 2, 128, 8, n_chunks=32)
    ids, Ks, Vs = fill(pool, [37, 8], rng)
    q = np.zeros((2, 8, 128), np.uint16)
    rc, out = pool.decode(ids, q)
    assert rc == 0
    for b in range(2):
        mean = f64(Vs[b]).mean(axis=0)                       # [Hkv, D]
        for h in range(8):
            assert np.abs(out[b, h] - mean[h // 4]).max() <= 1e-13
    pool.close()


def pin_constant_v(lib):
    """All V rows equal to c: the weights sum to one, so the output is c."""
    rng = np.random.default_rng(6)
    pool = make_pool(lib, 8, 8, 64, 16)
    c = W.normal_bf16(rng, (8, 64))
    L = 77
    V = np.broadcast_to(c, (L, 8, 64)).copy()
    K = W.normal_bf16(rng, (L, 8, 64))
    ids, _, _ = fill(pool, [L], rng, k=[K], v=[V])
    q = W.normal_bf16(rng, (1, 8, 64))
    rc, out = pool.decode(ids, q)
    assert rc == 0
    assert np.abs(out[0] - f64(c)).max() <= 1e-14
    pool.close()


def pin_weights_sum_to_one(lib):
    rng = np.random.default_rng(7)
    pool = make_pool(lib, 8, 8, 64, 16)
    ids, _, _ = fill(pool, [200, 3], rng)
    q = W.normal_bf16(rng, (8, 64))
    for tid in ids:
        for h in (0, 5):
            w = pool.weights(tid, q[h], h)
            assert (w >= 0).all()
            assert abs(w.sum() - 1.0) <= 1e-14
    pool.close()


def pin_two_token_logistic(lib):
    """Two tokens, q = 8 e_0, K_0 = x e_0, K_1 = 0, scale = 1/sqrt(64) = 1/8: scores are (x, 0), so the
    weights are the logistic function of x and the output is w V_0 + (1 - w) V_1. Also checks that an
    explicit scale replaces the default."""
    rng = np.random.default_rng(8)
    for x in (0.5, -2.0, 3.0):
        pool = make_pool(lib, 2, 2, 64, 16)
        K = np.zeros((2, 2, 64), np.float32)
        K[0, :, 0] = x
        V = rng.standard_normal((2, 2, 64)).astype(np.float32)
        Kb, Vb = W.bf16_bits_from_f32(K), W.bf16_bits_from_f32(V)
        ids, _, _ = fill(pool, [2], rng, k=[Kb], v=[Vb])
        qf = np.zeros((1, 2, 64), np.float32)
        qf[0, :, 0] = 8.0
        q = W.bf16_bits_from_f32(qf)
        rc, out = pool.decode(ids, q)
        assert rc == 0
        w = 1.0 / (1.0 + math.exp(-x))
        ref = w * f64(Vb[0]) + (1 - w) * f64(Vb[1])
        assert np.abs(out[0] - ref).max() <= 1e-14
        rc, out2 = pool.decode(ids, q, scale=0.25)          # scores (2x, 0)
        w2 = 1.0 / (1.0 + math.exp(-2.0 * x))
        ref2 = w2 * f64(Vb[0]) + (1 - w2) * f64(Vb[1])
        assert rc == 0 and np.abs(out2[0] - ref2).max() <= 1e-14
        pool.close()


def pin_dominant_key(lib):
    """One key aligned with q, all others orthogonal to q: the output tends to that key's V row with
    error at most (L-1) e^{-ds} * max|V_i - V_j|. The dominant key is the NEWEST token."""
    rng = np.random.default_rng(9)
    D, L = 64, 50
    pool = make_pool(lib, 1, 1, D, 16)
    K = np.zeros((L, 1, D), np.float32)
    K[:, 0, 1:] = rng.standard_normal((L, D - 1))
    K[L - 1, 0, 0] = 32.0                                    # score = 32 * 16 / 8 = 64 vs 0
    V = rng.standard_normal((L, 1, D)).astype(np.float32)
    Kb, Vb = W.bf16_bits_from_f32(K), W.bf16_bits_from_f32(V)
    ids, _, _ = fill(pool, [L], rng, k=[Kb], v=[Vb])
    qf = np.zeros((1, 1, D), np.float32)
    qf[0, 0, 0] = 16.0
    rc, out = pool.decode(ids, W.bf16_bits_from_f32(qf))
    assert rc == 0
    spread = np.abs(f64(Vb)).max() * 2
    assert np.abs(out[0, 0] - f64(Vb[L - 1, 0])).max() <= (L - 1) * math.exp(-64.0) * spread + 1e-15
    pool.close()


def pin_shift_invariance(lib):
    """Adding the same vector u to every K row shifts all scores equally and leaves the output
    unchanged. K and u live on a coarse power-of-two grid so K + u is exact in bf16."""
    rng = np.random.default_rng(10)
    D, L = 64, 40
    K = rng.integers(-8, 9, size=(L, 2, D)).astype(np.float32) / 4.0
    u = rng.integers(-8, 9, size=(1, 2, D)).astype(np.float32) / 4.0
    V = rng.standard_normal((L, 2, D)).astype(np.float32)
    q = W.normal_bf16(rng, (1, 4, D))
    outs = []
    for Kx in (K, K + u):
        pool = make_pool(lib, 4, 2, D, 16)
        ids, _, _ = fill(pool, [L], rng, k=[W.bf16_bits_from_f32(Kx)], v=[W.bf16_bits_from_f32(V)])
        rc, out = pool.decode(ids, q)
        assert rc == 0
        outs.append(out)
        pool.close()
    assert np.abs(outs[0] - outs[1]).max() <= 1e-12
    assert np.abs(outs[0]).max() > 1e-3


def pin_gqa_grouping(lib):
    """q heads of one group set equal give equal outputs; equal q heads in different groups (with
    different K/V) give different outputs; GQA equals MHA over kv heads repeated G times."""
    rng = np.random.default_rng(11)
    Hq, Hkv, D, L = 8, 2, 64, 45
    pool = make_pool(lib, Hq, Hkv, D, 16)
    ids, Ks, Vs = fill(pool, [L], rng)
    qrow = W.normal_bf16(rng, (D,))
    q = np.broadcast_to(qrow, (1, Hq, D)).copy()
    rc, out = pool.decode(ids, q)
    assert rc == 0
    for h in (1, 2, 3):
        assert np.array_equal(out[0, 0], out[0, h])
    for h in (5, 6, 7):
        assert np.array_equal(out[0, 4], out[0, h])
    assert np.abs(out[0, 0] - out[0, 4]).max() > 1e-3
    mha = make_pool(lib, Hq, Hq, D, 16)
    ids2, _, _ = fill(mha, [L], rng, k=[np.repeat(Ks[0], 4, axis=1)], v=[np.repeat(Vs[0], 4, axis=1)])
    rc, out2 = mha.decode(ids2, q)
    assert rc == 0 and np.array_equal(out, out2)
    pool.close(); mha.close()


def pin_chunked_equals_twin_and_online(lib):
    """Reading through the chunk table and byte image gives bit-identical results to the dense twin
    built straight from the append stream (pins translation + layout against each other); merging
    per-chunk partial softmaxes equals the two-pass result up to rounding."""
    cfg = W.CONFIGS["tiny"]
    st = W.draw_step(cfg)
    pool = OraclePool(cfg.n_chunks, cfg.chunk_bytes, 0, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                      cfg.batch, cfg.max_slots, None, True, lib)
    ids = []
    for b in range(cfg.batch):
        rc, tid = pool.tensor_create(cfg.max_tokens)
        assert rc == 0
        cid = st.placement.chunk_ids[b]
        assert pool.map_chunks(tid, 0, len(cid), cid) == 0
        assert pool.append([tid], st.k_hist[b], st.v_hist[b], [int(st.lens[b]) - 1]) == 0
        ids.append(tid)
    assert pool.append(ids, st.k_new, st.v_new) == 0
    rc0, a = pool.decode(ids, st.q, mode=MODE_CHUNKED)
    rc1, b_ = pool.decode(ids, st.q, mode=MODE_TWIN)
    rc2, c = pool.decode(ids, st.q, mode=MODE_ONLINE)
    assert rc0 == rc1 == rc2 == 0
    assert np.array_equal(a, b_)
    assert np.abs(a - c).max() <= 1e-12
    assert pool.check_invariants() == 0
    pool.close()


def pin_layout_bytes(lib):
    """The byte image after an append holds each value at the offset the chunk layout defines:
    ((h*2 + plane)*T_c + r)*D*2 + d*2. Offsets below are worked out by hand for the Tiny geometry
    (Hkv 8, D 64, T_c 16)."""
    rng = np.random.default_rng(12)
    pool = make_pool(lib, 8, 8, 64, 16)
    L = 22
    ids, Ks, Vs = fill(pool, [L], rng, chunk_perm=[9, 3])   # slot 0 -> chunk 3, slot 1 -> chunk 9
    c0 = pool.chunk_bytes_of(3).view(np.uint16)
    c1 = pool.chunk_bytes_of(9).view(np.uint16)
    # token 5, kv head 3, V plane, dim 7: byte ((3*2+1)*16+5)*128 + 14 = 14990 -> u16 index 7495
    assert c0[7495] == Vs[0][5, 3, 7]
    # token 5, kv head 3, K plane, dim 0: byte ((3*2+0)*16+5)*128 = 12928 -> 6464
    assert c0[6464] == Ks[0][5, 3, 0]
    # token 21 = slot 1 row 5, kv head 0, K plane, dim 63: byte (0*16+5)*128 + 126 = 766 -> 383
    assert c1[383] == Ks[0][21, 0, 63]
    # token 16 = slot 1 row 0, kv head 7, V plane, dim 1: byte ((7*2+1)*16)*128 + 2 = 30722 -> 15361
    assert c1[15361] == Vs[0][16, 7, 1]
    # rows never written stay zero in the oracle's image
    assert c1[(0 * 16 + 6) * 64] == 0
    pool.close()


def pin_remap_and_roundtrip_invariance(lib):
    """Offloading a request's chunks and fetching them into different physical chunks changes the
    table but not one bit of the attention output; migrated bytes are identical."""
    rng = np.random.default_rng(13)
    pool = make_pool(lib, 8, 8, 64, 16, n_chunks=32, n_host=8)
    ids, _, _ = fill(pool, [70, 40], rng)
    q = W.normal_bf16(rng, (2, 8, 64))
    rc, before = pool.decode(ids, q)
    tab0, _ = pool.table(ids[0])
    img0 = [pool.chunk_bytes_of(c) for c in tab0[:5]]
    assert pool.offload(ids[0], 0, 5) == 0
    rcx, _ = pool.decode(ids, q)
    assert rcx == -5                                          # not resident
    tabh, _ = pool.table(ids[0])
    assert list(tabh[:5]) == [-2, -3, -4, -5, -6]
    for i in range(5):
        assert np.array_equal(pool.host_slot_bytes(i), img0[i])
    o, s, _, _ = pool.owner_state()
    free = [c for c in range(32) if s[c] == 0 and c not in set(tab0[:5])][:5]
    assert pool.fetch(ids[0], 0, 5, free) == 0
    tab1, _ = pool.table(ids[0])
    assert list(tab1[:5]) == free and not set(free) & set(tab0[:5])
    for i in range(5):
        assert np.array_equal(pool.chunk_bytes_of(free[i]), img0[i])
    rc, after = pool.decode(ids, q)
    assert rc == 0 and np.array_equal(before, after)
    assert pool.check_invariants() == 0
    pool.close()


def pin_allocator_order_and_inflation(lib):
    """Pool-chosen chunks: lowest free KV-owned id first; with inflation allowed, then the lowest
    free activation-owned ids, which change owner; busy activation chunks are never taken."""
    owner = np.array([0, 1, 0, 1, 1, 0, 1, 0], np.uint8)
    pool = make_pool(lib, 8, 8, 64, 16, n_chunks=8, owner=owner, max_slots=8)
    rc, t = pool.tensor_create(128)
    assert pool.set_act_busy([3], 1) == 0
    assert pool.map_chunks(t, 0, 3) == 0
    assert list(pool.table(t)[0][:3]) == [0, 2, 5]
    assert pool.map_chunks(t, 3, 2) == -2                     # only one KV chunk left, no inflation
    assert list(pool.table(t)[0][3:5]) == [-1, -1]            # failed call changed nothing
    assert pool.map_chunks(t, 3, 3, None, 1) == 0             # 7 (KV), then 1, 4 (ACT; 3 is busy)
    assert list(pool.table(t)[0][3:6]) == [7, 1, 4]
    o, s, mt, ms = pool.owner_state()
    assert list(o) == [0, 0, 0, 1, 0, 0, 1, 0]
    assert list(s) == [1, 1, 1, 2, 1, 1, 0, 1]
    assert pool.map_chunks(t, 6, 2, None, 1) == -2            # one free ACT chunk (6) is not enough
    assert pool.transfer([3], 0) == -3                        # busy chunk cannot change owner
    assert pool.check_invariants() == 0
    pool.close()


def pin_unmap_rules(lib):
    """Unmapping undoes a speculative pre-map (Sec. 3.1): only slots behind the live tokens may go;
    their chunks are FREE again, their entries empty, a host copy in the tail gives its host slot
    back. A refused call changes nothing."""
    Tc = 16
    pool = make_pool(lib, 8, 8, 64, Tc, n_chunks=8, n_host=2, max_tensors=2, max_slots=6)
    _, t = pool.tensor_create(6 * Tc)
    assert pool.map_chunks(t, 0, 4, [5, 1, 6, 2]) == 0              # slots 0..3 -> chunks 5, 1, 6, 2
    tok = np.zeros((Tc + 1, 8, 64), np.uint16)
    assert pool.append([t], tok, tok, [Tc + 1]) == 0                 # 17 tokens: slots 0 and 1 are live
    before = [a.copy() for a in pool.owner_state()], pool.table(t)[0].copy()

    def unchanged():
        now = pool.owner_state()
        return all(np.array_equal(a, b) for a, b in zip(before[0], now)) and np.array_equal(before[1], pool.table(t)[0])

    assert pool.unmap_chunks(t, 1, 2) == -1 and unchanged()          # slot 1 holds token 16
    assert pool.unmap_chunks(t, 0, 1) == -1 and unchanged()
    assert pool.unmap_chunks(t, 3, 2) == -4 and unchanged()          # slot 4 has no chunk
    assert pool.unmap_chunks(t, 4, 3) == -6 and unchanged()          # past the tensor's 6 slots
    assert pool.unmap_chunks(t, 2, -1) == -1 and pool.unmap_chunks(7, 2, 1) == -1
    assert pool.unmap_chunks(t, 5, 0) == 0 and unchanged()
    # the pre-mapped tail goes: slot 3 (chunk 2) first, then slot 2 (chunk 6) after a trip to the host
    assert pool.unmap_chunks(t, 3, 1) == 0
    o, s, mt, ms = pool.owner_state()
    assert s[2] == 0 and mt[2] == -1 and ms[2] == -1 and o[2] == 0
    assert list(pool.table(t)[0]) == [5, 1, 6, -1, -1, -1] and pool.table(t)[1] == Tc + 1
    assert pool.offload(t, 2, 1) == 0
    assert list(pool.table(t)[0])[2] == -2 and pool.host_slots()[0][0] == t and pool.owner_state()[1][6] == 0
    assert pool.unmap_chunks(t, 2, 1) == 0
    assert list(pool.table(t)[0]) == [5, 1, -1, -1, -1, -1]
    th, ts = pool.host_slots()
    assert (th == -1).all() and (ts == -1).all()                     # the host slot is free again
    o, s, mt, ms = pool.owner_state()
    assert list(s) == [0, 1, 0, 0, 0, 1, 0, 0] and mt[5] == t and ms[1] == 1
    # the freed chunks are what the pool hands out next (lowest id first), so they really are FREE
    assert pool.map_chunks(t, 2, 2) == 0 and list(pool.table(t)[0])[2:4] == [0, 2]
    # a tensor with no token may lose every slot
    _, u = pool.tensor_create(2 * Tc)
    assert pool.map_chunks(u, 0, 2) == 0 and pool.unmap_chunks(u, 0, 2) == 0
    assert list(pool.table(u)[0]) == [-1, -1]
    assert pool.check_invariants() == 0
    pool.close()


def pin_act_busy_both_ways(lib):
    """The stand-in for live activations (Sec. 2.2.1 step 2: only chunks of inactive activation
    tensors can be lent): busy = 1 takes FREE activation chunks out of reach, busy = 0 gives BUSY
    ones back, after which they can change sides and be mapped. Wrong state or owner: refused,
    nothing changed."""
    owner = np.array([0, 1, 1, 1, 0, 1], np.uint8)
    pool = make_pool(lib, 8, 8, 64, 16, n_chunks=6, owner=owner, max_tensors=2, max_slots=6)
    assert pool.set_act_busy([1, 3], 1) == 0
    assert list(pool.owner_state()[1]) == [0, 2, 0, 2, 0, 0]
    assert pool.set_act_busy([2], 0) == -1                           # FREE, not BUSY
    assert pool.set_act_busy([1, 2], 0) == -1                        # second id is not BUSY: nothing changes
    assert list(pool.owner_state()[1]) == [0, 2, 0, 2, 0, 0]
    assert pool.set_act_busy([0], 0) == -3 and pool.set_act_busy([0], 1) == -3   # KV-owned
    assert pool.set_act_busy([6], 0) == -6 and pool.set_act_busy([-1], 1) == -6
    assert pool.set_act_busy([1, 1], 0) == -1                        # the same id twice
    assert pool.set_act_busy([1], 1) == -3                           # already BUSY
    assert pool.transfer([1], 0) == -3                               # a BUSY chunk cannot change sides
    _, t = pool.tensor_create(6 * 16)
    assert pool.map_chunks(t, 0, 5, None, 1) == -2                   # free: 0, 4 (KV), 2, 5 (ACT) = 4 < 5
    assert pool.set_act_busy([3, 1], 0) == 0
    o, s, mt, ms = pool.owner_state()
    assert list(s) == [0, 0, 0, 0, 0, 0] and list(o) == [0, 1, 1, 1, 0, 1] and (mt == -1).all()
    assert pool.transfer([1], 0) == 0 and pool.owner_state()[0][1] == 0          # now it can
    assert pool.map_chunks(t, 0, 5, None, 1) == 0                    # KV 0, 1, 4, then ACT 2, 3
    assert list(pool.table(t)[0])[:5] == [0, 1, 4, 2, 3]
    assert pool.set_act_busy([2], 0) == -3                           # lent to KV: no longer on the activation side
    assert pool.check_invariants() == 0
    pool.close()


def pin_inflation_walkthrough(lib, path):
    """Replays the inflation / deflation walk-through restated in tests/golden."""
    owner = np.array([0, 0, 0, 0, 1, 1, 1, 1], np.uint8)
    pool = make_pool(lib, 8, 8, 64, 16, n_chunks=8, owner=owner, max_tensors=16, max_slots=4)
    tensors = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        _, action, expect, fkv, fact, mapped = [x.strip() for x in line.split("|")]
        words = action.split()
        n = int(words[1])
        if words[0] in ("fill_kv", "map_new"):
            flags = 1 if (len(words) > 2 and words[2] == "inflate") else 0
            rc, t = pool.tensor_create(16 * n)
            assert rc == 0
            rc = pool.map_chunks(t, 0, n, None, flags)
            if rc == 0:
                tensors.append(t)
            else:
                pool.tensor_destroy(t)
        elif words[0] == "finish_newest":
            rc = 0
            for _ in range(n):
                rc |= pool.tensor_destroy(tensors.pop())
        elif words[0] == "transfer_free_to_act":
            o, s, _, _ = pool.owner_state()
            free = [c for c in range(8) if o[c] == 0 and s[c] == 0][:n]
            rc = pool.transfer(free, 1)
        else:
            raise AssertionError(action)
        assert (rc == 0) == (expect == "ok") and (rc == -2) == (expect == "oom"), (line, rc)
        o, s, _, _ = pool.owner_state()
        assert int(((o == 0) & (s == 0)).sum()) == int(fkv), line
        assert int(((o == 1) & (s == 0)).sum()) == int(fact), line
        assert int((s == 1).sum()) == int(mapped), line
        assert pool.check_invariants() == 0
    pool.close()


def pin_best_fit_is_the_arg_min(lib):
    """Sec. 2.1.2: among the available tensors with size >= s the smallest is taken (brute force
    over the sizes here; equal sizes: lowest handle, this build's reading). The mapping of the
    chosen tensor is kept as it is; with no fitting tensor a fresh one is mapped on demand."""
    rng = np.random.default_rng(7)
    Tc = 16
    for trial in range(30):
        pool = make_pool(lib, 8, 8, 64, Tc, n_chunks=64, n_host=4, max_tensors=12, max_slots=8)
        n_t = int(rng.integers(1, 9))
        slots = rng.integers(0, 7, size=n_t)                   # mapped slots per tensor; equal sizes are likely
        tables = []
        for i in range(n_t):
            rc, t = pool.tensor_create(8 * Tc)
            assert rc == 0 and t == i
            assert pool.map_chunks(t, 0, int(slots[i])) == 0
            tables.append(pool.table(t)[0].copy())
        released = sorted(rng.choice(n_t, size=int(rng.integers(0, n_t + 1)), replace=False).tolist())
        for t in released:
            assert pool.release(t) == 0
            assert pool.is_released(t) == 1 and pool.table(t)[1] == 0
            assert np.array_equal(pool.table(t)[0], tables[t])          # the mapping is retained
        s = int(rng.integers(0, 7 * Tc))
        sizes = {t: int(slots[t]) * Tc for t in released}
        feasible = [t for t in released if sizes[t] >= s]
        rc, got = pool.acquire(s, 8 * Tc)
        assert rc == 0
        if feasible:
            smallest = min(sizes[t] for t in feasible)
            want = min(t for t in feasible if sizes[t] == smallest)
            assert got == want, (trial, s, sizes, got, want)
            assert pool.is_released(got) == 0
            assert np.array_equal(pool.table(got)[0], tables[got])      # no mapping changed
        else:
            assert got == n_t                                           # lowest unused handle
            need = -(-s // Tc)
            tab = pool.table(got)[0]
            assert (tab[:need] >= 0).all() and (tab[need:] == -1).all()
            assert len(set(tab[:need].tolist())) == need
        assert pool.check_invariants() == 0
        pool.close()


def pin_release_acquire_premap_rules(lib):
    """A released tensor keeps only its leading mapped run, takes no request call, and is the first
    source of chunks when on-demand mapping runs short (smallest available tensor first, from its
    tail); pre-mapping gives exactly the requests about to open an empty slot one chunk each."""
    Tc = 16
    pool = make_pool(lib, 8, 8, 64, Tc, n_chunks=10, n_host=4, max_tensors=6, max_slots=8)
    _, a = pool.tensor_create(8 * Tc)
    _, b = pool.tensor_create(8 * Tc)
    assert pool.map_chunks(a, 0, 3) == 0 and pool.map_chunks(b, 0, 5) == 0      # a: 0,1,2  b: 3..7
    tok = np.zeros((40, 8, 64), np.uint16)
    assert pool.append([a], tok, tok, [40]) == 0
    assert pool.offload(a, 1, 1) == 0                                            # a: 0, host, 2
    assert pool.release(a) == 0
    assert list(pool.table(a)[0][:3]) == [0, -1, -1] and pool.table(a)[1] == 0   # run of 1 kept, rest given back
    th, _ = pool.host_slots()
    assert (th == -1).all()
    for call in (lambda: pool.map_chunks(a, 1, 1), lambda: pool.append([a], tok, tok, [1]),
                 lambda: pool.decode([a], np.zeros((1, 8, 64), np.uint16))[0], lambda: pool.release(a),
                 lambda: pool.offload(a, 0, 1), lambda: pool.premap_next([a])[0]):
        assert call() == -1
    assert pool.release(b) == 0
    # 10 chunks: 0 (a), 3..7 (b) mapped; free: 1, 2, 8, 9. A request for 7 slots fits no released tensor:
    # free chunks 1, 2, 8, 9 first, then from the smallest released tensor (a: chunk 0), then b's tail (7, 6)
    rc, c = pool.acquire(7 * Tc, 8 * Tc)
    assert rc == 0 and c == 2
    assert list(pool.table(c)[0][:7]) == [1, 2, 8, 9, 0, 7, 6]
    assert list(pool.table(a)[0][:1]) == [-1] and list(pool.table(b)[0][:5]) == [3, 4, 5, -1, -1]
    assert pool.acquire(4 * Tc, 8 * Tc)[0] == -2                                 # 3 chunks left in b, none free
    rc, d = pool.acquire(2 * Tc, 8 * Tc)
    assert rc == 0 and d == b and list(pool.table(b)[0][:3]) == [3, 4, 5]        # b (3 slots) fits; a (0) does not
    # pre-mapping
    assert pool.tensor_destroy(c) == 0
    assert pool.append([b], tok, tok, [32]) == 0                                 # b: 2 full slots of 3 -> next slot is mapped
    rc, e = pool.acquire(0, 8 * Tc)
    assert rc == 0 and e == a                                                    # a (size 0) is the best fit for nothing
    rc, n = pool.premap_next([b, e])
    assert (rc, n) == (0, 1) and pool.table(e)[0][0] == 0 and pool.table(b)[0][3] == -1
    assert pool.premap_next([b, e]) == (0, 0)
    assert pool.append([b], tok, tok, [16]) == 0
    rc, n = pool.premap_next([b, e])
    assert (rc, n) == (0, 1) and pool.table(b)[0][3] == 1
    assert pool.check_invariants() == 0
    pool.close()


def pin_premap_ahead_rules(lib):
    """Pre-mapping with a longer view: exactly the empty slots that the next tokens_ahead tokens of
    each listed tensor fall into get a chunk (hand-worked case with the chunk ids written out); one
    token ahead is the plain pre-mapping call; on random states the count equals the one taken from
    the tables in this test, and afterwards that many tokens can be appended with no further mapping."""
    Tc = 16
    pool = make_pool(lib, 8, 8, 64, Tc, n_chunks=9, n_host=0, max_tensors=4, max_slots=8)
    _, a = pool.tensor_create(8 * Tc)
    _, b = pool.tensor_create(8 * Tc)
    _, c = pool.tensor_create(24)                                                # two slots at most
    assert pool.map_chunks(a, 0, 2) == 0 and pool.map_chunks(b, 0, 2) == 0 and pool.map_chunks(c, 0, 1) == 0
    tok = np.zeros((32, 8, 64), np.uint16)
    assert pool.append([a], tok, tok, [20]) == 0 and pool.append([b], tok, tok, [32]) == 0
    assert pool.append([c], tok, tok, [5]) == 0
    # a: tokens 20..31 stay in slot 1 (mapped); b: 32..43 open slot 2; c: 5..16 reach into slot 1
    assert pool.premap_ahead([a, b, c], 12) == (0, 2)
    assert list(pool.table(a)[0][:3]) == [0, 1, -1] and list(pool.table(b)[0][:4]) == [2, 3, 5, -1]
    assert list(pool.table(c)[0]) == [4, 6]
    assert pool.premap_ahead([a], 13) == (0, 1) and list(pool.table(a)[0][:4]) == [0, 1, 7, -1]   # token 32 is in slot 2
    assert pool.premap_ahead([c], 1000) == (0, 0)                                # nothing beyond max_tokens
    assert pool.premap_ahead([a], 0)[0] == -1 and pool.premap_ahead([a, a], 4)[0] == -1
    before = [list(pool.table(t)[0]) for t in (a, b, c)]
    assert pool.premap_ahead([b, a], 40)[0] == -2                                # b needs 2, a 1: only chunk 8 is free
    assert [list(pool.table(t)[0]) for t in (a, b, c)] == before and pool.check_invariants() == 0
    pool.close()
    rng = np.random.default_rng(77)
    for trial in range(30):
        Tc = int(rng.choice([4, 16]))
        pools = [make_pool(lib, 2, 2, 64, Tc, n_chunks=120, n_host=0, max_tensors=6, max_slots=12) for _ in range(2)]
        ids, lens, maxes = [], [], []
        for i in range(5):
            mx = int(rng.integers(1, 12 * Tc + 1))
            L = int(rng.integers(0, mx + 1))
            mapped = min(-(-mx // Tc), -(-L // Tc) + int(rng.integers(0, 3)))    # sometimes slots are mapped already
            for q in pools:
                _, t = q.tensor_create(mx)
                assert q.map_chunks(t, 0, mapped) == 0
                z = np.zeros((L, 2, 64), np.uint16)
                assert q.append([t], z, z, [L]) == 0
            ids.append(t); lens.append(L); maxes.append(mx)
        k = int(rng.integers(1, 3 * Tc))
        # one token ahead is the plain call
        assert pools[0].premap_ahead(ids, 1) == pools[1].premap_next(ids)
        assert all(np.array_equal(pools[0].table(t)[0], pools[1].table(t)[0]) for t in ids)
        # k ahead: count from the tables
        want = 0
        for t, L, mx in zip(ids, lens, maxes):
            tab = pools[0].table(t)[0]
            slots = {tok_ // Tc for tok_ in range(L, min(L + k, mx))}
            want += sum(1 for s_ in slots if tab[s_] == -1)
        assert pools[0].premap_ahead(ids, k) == (0, want)
        for step in range(k):
            live = [t for t, L, mx in zip(ids, lens, maxes) if L + step < mx]
            z = np.zeros((len(live), 2, 64), np.uint16)
            assert pools[0].append(live, z, z) == 0
        assert pools[0].check_invariants() == 0
        for q in pools:
            q.close()


def pin_slo_buffer_trace(lib, path):
    """Replays the hand-worked trace of the logical buffer scaling (Sec. 2.3.2) in tests/golden, then
    checks that a shrunk logical buffer refuses offloads without evicting what is stored."""
    pool = make_pool(lib, 8, 8, 64, 16, n_chunks=80, n_host=64, max_tensors=4, max_slots=70)
    assert pool.slo_observe(1.0, 1.0)[0] == -1                       # not configured yet
    assert pool.slo_configure(1000.0, 50.0, 2.0, 5, 3) == 0
    assert pool.logical_host_slots() == 64
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        it, ttft, tpot, want = [x.strip() for x in line.split("|")[:4]]
        rc, got = pool.slo_observe(float(ttft), float(tpot))
        assert rc == 0 and got == int(want) == pool.logical_host_slots(), (line, got)
    # down to nothing and up again: floor(size / 2) ... 1 -> 0, then 0 grows to 2
    sizes = []
    for _ in range(8):
        for _ in range(3):
            rc, got = pool.slo_observe(0.0, 99.0)
        sizes.append(got)
    assert sizes == [32, 16, 8, 4, 2, 1, 0, 0]
    for _ in range(3):
        rc, got = pool.slo_observe(5000.0, 0.0)
    assert got == 2
    # the logical size limits offloads, and shrinking it evicts nothing
    _, t = pool.tensor_create(70 * 16)
    assert pool.map_chunks(t, 0, 6) == 0
    tok = np.zeros((96, 8, 64), np.uint16)
    assert pool.append([t], tok, tok, [96]) == 0
    assert pool.offload(t, 0, 3) == -8 and pool.offload(t, 0, 2) == 0          # two host slots usable
    assert pool.set_logical_host_slots(1) == 0
    th, _ = pool.host_slots()
    assert int((th >= 0).sum()) == 2                                             # still stored
    assert pool.offload(t, 2, 1) == -8
    assert pool.set_logical_host_slots(3) == 0 and pool.offload(t, 2, 1) == 0
    assert pool.set_logical_host_slots(65) == -6 and pool.set_logical_host_slots(-1) == -6
    assert pool.check_invariants() == 0
    pool.close()


ALL_PINS = [pin_sdpa_library, pin_single_token, pin_zero_query_is_mean, pin_constant_v,
            pin_weights_sum_to_one, pin_two_token_logistic, pin_dominant_key, pin_shift_invariance,
            pin_gqa_grouping, pin_chunked_equals_twin_and_online, pin_layout_bytes,
            pin_remap_and_roundtrip_invariance, pin_allocator_order_and_inflation, pin_best_fit_is_the_arg_min,
            pin_release_acquire_premap_rules, pin_unmap_rules, pin_act_busy_both_ways, pin_premap_ahead_rules]
