"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same seeded
inputs. Tables, owner/state arrays and migrated bytes bit-exact; bf16 attention output within
max-abs 2e-2 and mean-abs 2e-3 of the oracle."""
import numpy as np
import pytest
import torch

import paper_2506_15155_amd as E
import workloads as W
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def run_step(cfg, seed=None, keep_twin=False, split=None, owner_from_placement=True):
    st = W.draw_step(cfg, seed)
    B = H.Both(cfg, owner=st.placement.owner if cfg.act_fraction > 0 else None, keep_twin=keep_twin)
    ids = H.load_step(B, st)
    assert B.append(ids, st.k_new, st.v_new) == 0
    if split:
        E.ellm_pool_set_split_tokens(B.pool, split)
    rc, out = B.decode(ids, st.q)
    assert rc == 0
    rco, ref = B.orc.decode(ids, st.q)
    assert rco == 0
    B.compare_state()
    return B, st, ids, out, ref


def test_tiny_config_exhaustive(pool_mode):
    """Config 1 as stated: every output element, every table entry, every byte of every chunk."""
    cfg = W.CONFIGS["tiny"]
    st = W.draw_step(cfg)
    B = H.Both(cfg, keep_twin=True)
    poison = np.full(cfg.chunk_bytes // 2, H.POISON, np.uint16).view(np.uint8)
    for c in range(cfg.n_chunks):
        B.orc.chunk_set_bytes(c, poison)
    ids = H.load_step(B, st)
    assert B.append(ids, st.k_new, st.v_new) == 0
    rc, out = B.decode(ids, st.q)
    rco, ref = B.orc.decode(ids, st.q)
    assert rc == 0 and rco == 0
    H.check_close(out, ref, "tiny")
    B.compare_state()
    for c in range(cfg.n_chunks):      # appended rows landed exactly where the layout says, nothing else moved
        assert np.array_equal(B.chunk_bytes_dev(c), B.orc.chunk_bytes_of(c)), c
    lens = [E.ellm_tensor_get_table(B.pool, t)[1] for t in ids]
    assert lens == [int(x) for x in st.lens]
    B.close()


@pytest.mark.parametrize("split", [16, 64, 256, 4096])
def test_tiny_split_sizes(split):
    """One split per request up to sixteen: all within tolerance of the oracle and of each other."""
    B, st, ids, out, ref = run_step(W.CONFIGS["tiny"], split=split)
    H.check_close(out, ref, f"split {split}")
    E.ellm_pool_set_split_tokens(B.pool, 4096)
    rc, one = B.decode(ids, st.q)
    assert rc == 0
    assert np.abs(H.out_f64(out) - H.out_f64(one)).max() <= 2 ** -6   # bf16 rounding of nearly equal fp32 sums
    B.close()


def test_run_to_run_bitwise_determinism(pool_mode):
    B, st, ids, out, ref = run_step(W.CONFIGS["tiny"], split=32)
    for _ in range(3):
        rc, again = B.decode(ids, st.q)
        assert rc == 0 and torch.equal(out, again)
    B.close()


REDUCED = {
    # config-2 shapes, fewer and shorter requests: several chunks per request, ragged tails
    "llama8b_small": W.scaled(W.CONFIGS["llama8b"], batch=12, n_chunks=96, len_lo=64, len_hi=2500, lognormal_median=700),
    # config-3 shapes: 102 tokens per chunk with slack, half the pool busy activations
    "mha13b_small": W.scaled(W.CONFIGS["mha13b"], batch=6, n_chunks=160, len_lo=90, len_hi=900, max_tokens=1020),
    # config-5 shapes: group of 8
    "long70b_small": W.scaled(W.CONFIGS["long70b"], batch=3, n_chunks=48, len_lo=1500, len_hi=6000, max_tokens=6144),
}


@pytest.mark.parametrize("name", sorted(REDUCED))
def test_reduced_configs_elementwise(name, pool_mode):
    B, st, ids, out, ref = run_step(REDUCED[name])
    mx, mean = H.check_close(out, ref, name)
    print(f"{name}: max-abs {mx:.2e} mean-abs {mean:.2e}")
    B.close()


@pytest.mark.parametrize("name,split", [("llama8b_small", 128), ("llama8b_small", 1024), ("mha13b_small", 102),
                                        ("mha13b_small", 64), ("long70b_small", 512)])
def test_reduced_configs_other_partitions(name, split):
    B, st, ids, out, ref = run_step(REDUCED[name], split=split)
    H.check_close(out, ref, f"{name}/{split}")
    B.close()


@pytest.mark.parametrize("Hq,Hkv,D", [(12, 2, 128), (6, 2, 64), (3, 1, 128), (32, 2, 64), (5, 5, 64)])
def test_other_group_sizes(Hq, Hkv, D, pool_mode):
    """Group sizes that are not 1, 2, 4 or 8 are covered by several launches over the same K/V."""
    cfg = W.Config("g", 9, 5, Hq, Hkv, D, 24 * (2 * Hkv * D * 2), 64, 24 * 12, "uniform", 1, 24 * 12)
    if pool_mode == "driver" and cfg.chunk_bytes % 4096:
        pytest.skip("the driver maps whole 4 KiB pages: this chunk size cannot be a mapping unit")
    B, st, ids, out, ref = run_step(cfg, seed=77)
    H.check_close(out, ref, f"Hq{Hq}/Hkv{Hkv}")
    B.close()


def test_more_waves_per_head_than_the_lookup_table_holds():
    """With one 64-token tile per wave a batch of 40 requests makes about 900 waves per kv head: more
    than the byte table in the kernel arguments covers, so the waves find their request by searching
    the tile prefix sums instead."""
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=40, n_chunks=200, len_lo=1000, len_hi=2000, lognormal_median=1400)
    B, st, ids, out, ref = run_step(cfg, seed=61, split=64)
    n_split, S = E.ellm_decode_plan(B.pool, ids)
    assert S == 64 and int(n_split.sum()) > 512
    H.check_close(out, ref, "request search")
    E.ellm_pool_set_split_tokens(B.pool, 0)
    rc, auto = B.decode(ids, st.q)
    assert rc == 0
    H.check_close(auto, ref, "automatic cut, same batch")
    B.close()


def test_pool_in_driver_mapped_memory():
    """The paper's own mechanism underneath (Sec. 2.1.1, Sec. 3.2): every 2 MiB chunk of the pool is a
    physical allocation of its own, mapped by the driver into one virtual range in a shuffled order.
    The library sees one buffer, as always: append, fused append + decode and an offload / fetch
    round trip must behave exactly as in a plain allocation."""
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=6, n_chunks=40, len_lo=300, len_hi=1500, lognormal_median=700,
                   host_slots=4)
    st = W.draw_step(cfg, 31)
    B = H.Both(cfg, owner=st.placement.owner if cfg.act_fraction > 0 else None, driver_mapped=True)
    poison = np.full(cfg.chunk_bytes // 2, H.POISON, np.uint16).view(np.uint8)
    for c in range(cfg.n_chunks):
        B.orc.chunk_set_bytes(c, poison)
    ids = H.load_step(B, st)
    rc, out, ref = B.append_decode(ids, st.k_new, st.v_new, st.q)
    assert rc == 0
    H.check_close(out, ref, "driver-mapped pool, fused call")
    B.compare_state()
    tab, _ = E.ellm_tensor_get_table(B.pool, ids[0])
    resident = [int(c) for c in tab if c >= 0]
    for c in resident:     # bytes of the chunks, history and new rows, as the oracle has them
        assert np.array_equal(B.chunk_bytes_dev(c), B.orc.chunk_bytes_of(c)), c
    assert B.offload(ids[0], 0, 1) == 0
    assert B.fetch(ids[0], 0, 1) == 0
    assert E.ellm_pool_sync(B.pool) == 0
    B.compare_state()
    rc, again = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(out, again)
    B.close()


def test_batch_larger_than_one_launch(pool_mode):
    """More requests than one launch's argument block describes (128)."""
    cfg = W.Config("wide", 8, 300, 8, 2, 64, 16 * (2 * 2 * 64 * 2), 700, 32, "uniform", 1, 32)
    B, st, ids, out, ref = run_step(cfg, seed=5)
    H.check_close(out, ref, "batch 300")
    B.close()


def test_closed_forms_on_gpu():
    cfg = W.scaled(W.CONFIGS["tiny"], batch=1)
    rng = np.random.default_rng(3)
    # L = 1: output is V[0] bit for bit
    B = H.Both(cfg, max_tensors=4)
    t = B.create(64)
    assert B.map(t, 0, 1, [7]) == 0
    k, v = W.normal_bf16(rng, (1, 8, 64)), W.normal_bf16(rng, (1, 8, 64))
    assert B.append([t], k, v) == 0
    q = W.normal_bf16(rng, (1, 8, 64))
    rc, out = B.decode([t], q)
    assert rc == 0 and np.array_equal(H.host_bits(out)[0], v[0])
    # constant V over 100 tokens: weights sum to one, so the output is that constant (to bf16 rounding)
    t2 = B.create(128)
    assert B.map(t2, 0, 7, [1, 60, 2, 59, 3, 58, 4]) == 0
    c = W.normal_bf16(rng, (8, 64))
    vv = np.broadcast_to(c, (100, 8, 64)).copy()
    kk = W.normal_bf16(rng, (100, 8, 64))
    assert B.append([t2], kk, vv, [100]) == 0
    rc, out = B.decode([t2], q)
    cf = W.f32_from_bf16_bits(c).astype(np.float64)
    assert rc == 0 and np.abs(H.out_f64(out)[0] - cf).max() <= np.abs(cf).max() * 2 ** -8
    # q = 0: arithmetic mean of V
    t3 = B.create(128)
    assert B.map(t3, 0, 3) == 0
    v3 = W.normal_bf16(rng, (37, 8, 64))
    assert B.append([t3], W.normal_bf16(rng, (37, 8, 64)), v3, [37]) == 0
    rc, out = B.decode([t3], np.zeros((1, 8, 64), np.uint16))
    mean = W.f32_from_bf16_bits(v3).astype(np.float64).mean(axis=0)
    assert rc == 0 and np.abs(H.out_f64(out)[0] - mean).max() <= 4e-3
    B.close()


def test_offload_fetch_remap_invariance_and_bytes(pool_mode):
    """Offload two requests' chunks, fetch them into other chunks: tables match the oracle, migrated
    bytes are identical (device before = host slot = device after), output bits do not change."""
    cfg = W.scaled(W.CONFIGS["tiny"], host_slots=40, batch=4)
    st = W.draw_step(cfg, seed=11)
    B = H.Both(cfg)
    poison = np.full(cfg.chunk_bytes // 2, H.POISON, np.uint16).view(np.uint8)
    for c in range(cfg.n_chunks):
        B.orc.chunk_set_bytes(c, poison)
    ids = H.load_step(B, st)
    assert B.append(ids, st.k_new, st.v_new) == 0
    rc, before = B.decode(ids, st.q)
    assert rc == 0
    for b in (0, 2):
        tab, _ = E.ellm_tensor_get_table(B.pool, ids[b])
        live = int((tab >= 0).sum())
        pre = [B.chunk_bytes_dev(int(c)) for c in tab[:live]]
        assert B.offload(ids[b], 0, live) == 0
        E.ellm_pool_sync(B.pool)
        tabh, _ = E.ellm_tensor_get_table(B.pool, ids[b])
        for i in range(live):
            hs = -int(tabh[i]) - 2
            assert np.array_equal(B.host_slot_bytes(hs), pre[i])
            assert np.array_equal(B.orc.host_slot_bytes(hs), pre[i])
        assert E.ellm_decode_attention(B.pool, ids, H.dev_bits(st.q), before.clone(), check=False) == E.ERR.NOT_RESIDENT
        # land in other chunks than before: take the highest free ids
        _, s, _, _ = E.ellm_pool_get_owner_state(B.pool)
        free = [c for c in range(cfg.n_chunks - 1, -1, -1) if s[c] == 0 and c not in set(int(x) for x in tab[:live])][:live]
        assert len(free) == live
        assert B.fetch(ids[b], 0, live, free) == 0
        E.ellm_pool_sync(B.pool)
        for i in range(live):
            assert np.array_equal(B.chunk_bytes_dev(free[i]), pre[i])
    B.compare_state()
    rc, after = B.decode(ids, st.q)
    assert rc == 0 and torch.equal(before, after)
    B.close()


FUSED_CASES = {
    "tiny": W.CONFIGS["tiny"],
    **REDUCED,
    "g3": W.Config("g3", 9, 5, 12, 4, 128, 24 * (2 * 4 * 128 * 2), 64, 24 * 12, "uniform", 1, 24 * 12),
    "g5_d64": W.Config("g5", 9, 6, 10, 2, 64, 40 * (2 * 2 * 64 * 2), 64, 40 * 8, "uniform", 1, 40 * 8),
}


@pytest.mark.parametrize("name", sorted(FUSED_CASES))
def test_fused_append_decode_equals_separate_calls(name, pool_mode):
    """ellm_kv_append_decode against ellm_kv_append + ellm_decode_attention on a twin pool: same
    output bits, same tables and lengths, same chunk bytes; and against the oracle."""
    cfg = FUSED_CASES[name]
    st = W.draw_step(cfg, seed=31)
    owner = st.placement.owner if cfg.act_fraction > 0 else None
    F = H.Both(cfg, owner=owner)
    S = H.Both(cfg, owner=owner, oracle=False, mode="table")     # the twin is always a plain pool
    ids = H.load_step(F, st)
    ids_s = H.load_step(S, st)
    assert ids == ids_s
    rc, out, ref = F.append_decode(ids, st.k_new, st.v_new, st.q)
    assert rc == 0
    assert S.append(ids, st.k_new, st.v_new) == 0
    rc, sep = S.decode(ids, st.q)
    assert rc == 0
    assert torch.equal(out, sep), "fused and separate calls disagree"
    H.check_close(out, ref, f"fused {name}")
    F.compare_state()
    for b, t in enumerate(ids):
        tab, ln = E.ellm_tensor_get_table(F.pool, t)
        assert ln == int(st.lens[b])
        for c in tab[tab >= 0]:
            assert np.array_equal(F.chunk_bytes_dev(int(c)), S.chunk_bytes_dev(int(c))), (b, int(c))
    # a second fused step on top (the row written by the first must be read back from the chunk)
    rng = np.random.default_rng(5)
    room = [b for b in range(cfg.batch) if int(st.lens[b]) % cfg.tokens_per_chunk != 0]
    sel = [ids[b] for b in room]
    if sel:
        k2 = W.normal_bf16(rng, (len(sel), cfg.n_kv_heads, cfg.head_dim))
        v2 = W.normal_bf16(rng, (len(sel), cfg.n_kv_heads, cfg.head_dim))
        q2 = W.normal_bf16(rng, (len(sel), cfg.n_q_heads, cfg.head_dim))
        rc, out2, ref2 = F.append_decode(sel, k2, v2, q2)
        assert rc == 0
        H.check_close(out2, ref2, f"fused {name}, second step")
        F.compare_state()
    F.close()
    S.close()


def test_fused_append_decode_errors_change_nothing():
    cfg = W.scaled(W.CONFIGS["tiny"], batch=2)
    B = H.Both(cfg, max_tensors=4)
    t = B.create(64)
    u = B.create(64)
    assert B.map(t, 0, 1) == 0
    one = np.zeros((2, 8, 64), np.uint16)
    k, q = H.dev_bits(one), H.dev_bits(one)
    out = torch.full_like(q, 123)
    # second request has no chunk: nothing may change for the first one either
    assert E.ellm_kv_append_decode(B.pool, [t, u], k, k, q, out, check=False) == E.ERR.UNMAPPED
    assert E.ellm_kv_append_decode(B.pool, [t, t], k, k, q, out, check=False) == E.ERR.INVALID
    assert E.ellm_kv_append_decode(B.pool, [t], None, k, q, out, check=False) == E.ERR.INVALID
    torch.cuda.synchronize()
    assert (out == 123).all()
    assert E.ellm_tensor_get_table(B.pool, t)[1] == 0
    B.compare_state()
    B.close()


def test_layerwise_fetch_under_attention(pool_mode):
    """Several layers in one pool, a third of the requests parked in host memory. Per step and layer:
    the fetch of the next layer's chunks is issued before this layer's attention, the offload of this
    layer's chunks right after it, and the freed chunks are reused at once by a scratch tensor. The
    side stream and the compute stream are ordered per chunk only, so any missing wait shows up as
    poison or stale rows. Checked against a twin pool that never migrates (same bits), the oracle
    (tolerance, tables, host bytes)."""
    n_layers = 3
    base = W.scaled(W.CONFIGS["llama8b"], batch=9, n_chunks=160, len_lo=300, len_hi=1400, lognormal_median=700,
                    host_slots=40)
    st = W.draw_step(base, seed=41, extra_slots=0)
    Bq, Tc = base.batch, base.tokens_per_chunk
    M = H.Both(base, max_tensors=n_layers * Bq + 1)
    T = H.Both(base, oracle=False, max_tensors=n_layers * Bq + 1, mode="table")
    rng = np.random.default_rng(43)
    free = list(rng.permutation(base.n_chunks).astype(np.int32))
    ids = []
    for l in range(n_layers):
        row = []
        for b in range(Bq):
            n = -(-int(st.lens[b]) // Tc)
            cid = np.array([free.pop() for _ in range(n)], np.int32)
            tm, tt = M.create(base.max_tokens), T.create(base.max_tokens)
            assert tm == tt
            assert M.map(tm, 0, n, cid) == 0 and T.map(tt, 0, n, cid) == 0
            k = W.normal_bf16(rng, (int(st.lens[b]) - 1, base.n_kv_heads, base.head_dim))
            v = W.normal_bf16(rng, (int(st.lens[b]) - 1, base.n_kv_heads, base.head_dim))
            assert M.append([tm], k, v, [int(st.lens[b]) - 1]) == 0 and T.append([tt], k, v, [int(st.lens[b]) - 1]) == 0
            row.append(tm)
        ids.append(row)
    scratch = M.create(Tc)
    T.create(Tc)
    parked = [0, 4, 7]
    lens = st.lens.copy() - 1
    n_slots = lambda b: -(-int(lens[b]) // Tc)
    for l in range(n_layers):
        for b in parked:
            assert M.offload(ids[l][b], 0, n_slots(b)) == 0
    M.compare_state()
    shape = (Bq, base.n_kv_heads, base.head_dim)
    for step in range(3):
        for b in parked:
            assert M.fetch(ids[0][b], 0, n_slots(b)) == 0
        for l in range(n_layers):
            if l + 1 < n_layers:
                for b in parked:                       # next layer's chunks start moving now
                    assert M.fetch(ids[l + 1][b], 0, n_slots(b)) == 0
            k1, v1 = W.normal_bf16(rng, shape), W.normal_bf16(rng, shape)
            q = W.normal_bf16(rng, (Bq, base.n_q_heads, base.head_dim))
            rc, out, ref = M.append_decode(ids[l], k1, v1, q)
            assert rc == 0
            rct, twin, _ = T.append_decode(ids[l], k1, v1, q)
            assert rct == 0
            assert torch.equal(out, twin), f"step {step} layer {l}: migrating pool differs from the twin"
            H.check_close(out, ref, f"step {step} layer {l}")
            for b in parked:                           # and this layer's go back to the host
                assert M.offload(ids[l][b], 0, -(-(int(lens[b]) + 1) // Tc)) == 0
            # reuse a chunk the offload has just freed: the copy must have read it before the append writes
            assert M.map(scratch, 0, 1) == 0
            junk = W.normal_bf16(rng, (5, base.n_kv_heads, base.head_dim))
            assert M.append([scratch], junk, junk, [5]) == 0
            assert E.ellm_tensor_destroy(M.pool, scratch, check=False) == 0 == M.orc.tensor_destroy(scratch)
            M.ids.remove(scratch)
            assert M.create(Tc) == scratch
        lens += 1
        E.ellm_pool_sync(M.pool)
        torch.cuda.synchronize()
        M.compare_state()
        th, sh = E.ellm_pool_get_host_slots(M.pool)
        for hs in np.flatnonzero(th >= 0)[:6]:          # parked bytes equal the oracle's image of them
            got, want = M.host_slot_bytes(int(hs)), M.orc.host_slot_bytes(int(hs))
            used = 2 * base.n_kv_heads * Tc * base.head_dim * 2
            t_id, t_slot = int(th[hs]), int(sh[hs])
            b = ids[t_id // Bq].index(t_id) if t_id in ids[t_id // Bq] else None
            rows = min(Tc, int(lens[b]) - t_slot * Tc)
            g = got[:used].reshape(base.n_kv_heads * 2, Tc, base.head_dim * 2)
            w = want[:used].reshape(base.n_kv_heads * 2, Tc, base.head_dim * 2)
            assert np.array_equal(g[:, :rows], w[:, :rows])
    M.close()
    T.close()


def test_request_turnover_best_fit_reuse(pool_mode):
    """Requests finish and are released with their chunks still mapped; new requests take the
    best-fitting released tensor (no table entry changes), write their prompt with a multi-token
    append over the previous owner's rows, pre-map one step ahead and decode. The previous
    owner's stale rows lie right behind the new length, so any read past the length shows."""
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=8, n_chunks=64, len_lo=200, len_hi=1900, lognormal_median=800)
    st = W.draw_step(cfg, seed=51)
    B = H.Both(cfg, max_tensors=12)
    ids = H.load_step(B, st)
    rc, out, ref = B.append_decode(ids, st.k_new, st.v_new, st.q)
    assert rc == 0
    H.check_close(out, ref, "before turnover")
    rng = np.random.default_rng(52)
    Tc = cfg.tokens_per_chunk
    live = list(ids)
    lens = {t: int(l) for t, l in zip(ids, st.lens)}
    for round_ in range(4):
        done = [live[i] for i in sorted(rng.choice(len(live), size=3, replace=False))]
        tables = {t: E.ellm_tensor_get_table(B.pool, t)[0].copy() for t in done}
        for t in done:
            assert B.release(t) == 0
            live.remove(t)
        for _ in range(3):
            prompt = int(rng.integers(1, 1500))
            rc, t = B.acquire(prompt, cfg.max_tokens, E.ELLM_MAP_ALLOW_INFLATE)
            assert rc == 0
            if t in tables:                        # a released tensor was reused: same chunks as before
                run = int((tables[t] >= 0).cumprod().sum())
                assert np.array_equal(E.ellm_tensor_get_table(B.pool, t)[0][:run], tables[t][:run])
                assert run * Tc >= prompt
            k = W.normal_bf16(rng, (prompt, cfg.n_kv_heads, cfg.head_dim))
            v = W.normal_bf16(rng, (prompt, cfg.n_kv_heads, cfg.head_dim))
            assert B.append([t], k, v, [prompt]) == 0
            live.append(t)
            lens[t] = prompt
        rc, n = B.premap_next(live, E.ELLM_MAP_ALLOW_INFLATE)
        assert rc == 0
        E.ellm_pool_flush_tables(B.pool)
        shape = (len(live), cfg.n_kv_heads, cfg.head_dim)
        k1, v1 = W.normal_bf16(rng, shape), W.normal_bf16(rng, shape)
        q = W.normal_bf16(rng, (len(live), cfg.n_q_heads, cfg.head_dim))
        rc, out, ref = B.append_decode(live, k1, v1, q)
        assert rc == 0, E.ellm_last_error()
        H.check_close(out, ref, f"turnover round {round_}")
        for t in live:
            lens[t] += 1
        B.compare_state()
    B.close()


def test_error_paths_launch_nothing():
    cfg = W.scaled(W.CONFIGS["tiny"], batch=2, host_slots=4)
    B = H.Both(cfg)
    t = B.create(64)
    q = H.dev_bits(np.zeros((1, 8, 64), np.uint16))
    out = torch.full_like(q, 123)
    assert E.ellm_decode_attention(B.pool, [t], q, out, check=False) == E.ERR.EMPTY
    assert E.ellm_kv_append(B.pool, [t], q, q, check=False) == E.ERR.UNMAPPED
    assert E.ellm_decode_attention(B.pool, [5], q, out, check=False) == E.ERR.INVALID
    torch.cuda.synchronize()
    assert (out == 123).all()
    B.close()
