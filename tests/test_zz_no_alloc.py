"""The entry point that allocates nothing, ellm_decode_attention_noalloc, through the C ABI against
ellm_decode_attention on the same pool: same output bits, on two calls in a row, the second over a
smaller batch; no device memory is allocated by the calls; sizes beyond the fixed workspace are
refused with an error and launch nothing."""
import numpy as np
import pytest
import torch

import paper_2506_15155_amd as E
import workloads as W
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def test_noalloc_decode_matches_the_allocating_entry_point():
    cfg = W.scaled(W.CONFIGS["llama8b"], batch=24, n_chunks=260, len_lo=64, len_hi=6000, lognormal_median=1500)
    st = W.draw_step(cfg, seed=71)
    B = H.Both(cfg)
    q = H.dev_bits(st.q)
    E.ellm_pool_prepare(B.pool)                  # device-side metadata created here, not in a later call
    ids = H.load_step(B, st)
    assert B.append(ids, st.k_new, st.v_new) == 0
    rc, want = B.decode(ids, st.q)
    assert rc == 0
    rco, ref = B.orc.decode(ids, st.q)
    assert rco == 0
    H.check_close(want, ref, "allocating entry point")
    got = torch.full_like(q, 77)
    small = torch.full_like(q[:5], 77)
    sub = [ids[b] for b in (20, 3, 11, 7, 0)]
    qs = q[[20, 3, 11, 7, 0]].contiguous()
    torch.cuda.synchronize()
    before = torch.cuda.mem_get_info()[0]        # free device memory as the driver sees it; torch allocates nothing below
    rc1 = E.ellm_decode_attention_noalloc(B.pool, ids, q, got, check=False)
    rc2 = E.ellm_decode_attention_noalloc(B.pool, sub, qs, small, check=False)   # second call, smaller input
    torch.cuda.synchronize()
    after = torch.cuda.mem_get_info()[0]
    assert rc1 == 0 and rc2 == 0, E.ellm_last_error()
    assert after == before, "the call changed the amount of free device memory"
    assert torch.equal(got, want)
    rc, want_small = B.decode(sub, st.q[[20, 3, 11, 7, 0]])
    assert rc == 0 and torch.equal(small, want_small)
    H.check_close(small, ref[[20, 3, 11, 7, 0]], "second, smaller call")
    B.compare_state()
    B.close()


def test_noalloc_decode_refuses_what_does_not_fit():
    # 64 q heads per kv head: one partial slot is 64 * 130 * 4 bytes, and the slots of one launch exceed 16 MiB
    cfg = W.Config("wide_group", 9, 4, 64, 1, 128, 64 * (2 * 1 * 128 * 2), 3000, 64 * 700, "uniform", 64 * 600, 64 * 700)
    st = W.draw_step(cfg, seed=3, with_values=False)
    dev = torch.zeros(cfg.n_chunks * cfg.chunk_bytes, dtype=torch.uint8, device="cuda")
    pool = E.ellm_pool_create(dev, None, cfg.chunk_bytes, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.batch, cfg.max_slots)
    ids = []
    kv = torch.zeros((int(st.lens.max()), 1, 128), dtype=torch.bfloat16, device="cuda")
    for b in range(cfg.batch):
        t = E.ellm_tensor_create(pool, cfg.max_tokens)
        E.ellm_tensor_map_chunks(pool, t, 0, len(st.placement.chunk_ids[b]), st.placement.chunk_ids[b])
        ids.append(t)
    q = torch.zeros((cfg.batch, 64, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 5.0)
    assert E.ellm_decode_attention_noalloc(pool, ids, q, out, check=False) == E.ERR.EMPTY
    for b in range(cfg.batch):
        E.ellm_kv_append(pool, [ids[b]], kv, kv, [int(st.lens[b])])
    n_split, _ = E.ellm_decode_plan(pool, ids)
    need = int(n_split[n_split > 1].sum()) * 64 * 130 * 4
    assert need > E.ELLM_NOALLOC_WORKSPACE_BYTES
    rc = E.ellm_decode_attention_noalloc(pool, ids, q, out, check=False)
    torch.cuda.synchronize()
    assert rc == E.ERR.RANGE and "fixed" in E.ellm_last_error()
    assert (out == 5.0).all()                                   # nothing was launched
    assert E.ellm_decode_attention(pool, ids, q, out, check=False) == 0      # the allocating entry point takes it
    torch.cuda.synchronize()
    assert (out == 0).all()
    E.ellm_pool_destroy(pool)
