"""Benchmark: decode attention + KV append over chunk-backed KV on one MI355X.

Workload (default): the Llama-3-8B-shaped configuration — 32 q / 8 kv heads, head_dim 128, bf16,
batch 64, context lengths lognormal (median 1k, clipped 64..8k), 2 MiB chunks shuffled in one
unified pool — for all 32 layers of such a model: every (layer, request) is a virtual KV tensor of
its own, so one step streams 32 different layers' K/V (about 13 GB) and the last-level cache cannot
serve the reads. One step = for every layer: map a chunk ahead for requests about to cross a
chunk boundary, append one token per request, decode-attend over the whole context.

Prints ONE JSON line: metric, value (whole-step GB/s of algorithmic bytes), ms_per_step, the workload in
`config`, `roofline` for the attention kernel (HIP-event time per launch against the 8 TB/s HBM peak, plus
measured read ceilings) and `cpu_baseline` (the fp64 CPU oracle timed on the host cores).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, public specification
COPY_CALIBRATION_BYTES = 1 << 30


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="llama8b", choices=["llama8b", "mha13b", "long70b", "tiny"])
    ap.add_argument("--layers", type=int, default=0, help="0 = the model's layer count for the shape")
    ap.add_argument("--split", type=int, default=0, help="override tokens per work item (0 = automatic)")
    ap.add_argument("--waves-percent", type=int, default=0,
                    help="waves per decode launch as a percentage of the library's choice, one wave per SIMD (0 = leave it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--event-stride", type=int, default=7, help="time every n-th attention launch with HIP events")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured read ceilings")
    ap.add_argument("--separate-calls", action="store_true",
                    help="ellm_kv_append then ellm_decode_attention instead of the fused ellm_kv_append_decode")
    ap.add_argument("--migration", action="store_true",
                    help="also time the elastic step: 25%% of the requests parked in pinned host memory, fetched and "
                         "offloaded every step, all at once and layer by layer under the attention")
    ap.add_argument("--turnover", action="store_true",
                    help="also time request turnover on the host: release + best-fit acquire against destroy + create + map")
    ap.add_argument("--pool-memory", default="malloc", choices=["malloc", "vmm"],
                    help="vmm: the pool's chunks are physical allocations of their own, mapped into one virtual range "
                         "by the driver in a shuffled order (the paper's mechanism) instead of one plain allocation")
    ap.add_argument("--placement", default="shuffled", choices=["shuffled", "contiguous"],
                    help="contiguous: every tensor gets consecutive chunk ids (what a kernel sees under the paper's "
                         "mechanism: contiguous virtual addresses)")
    ap.add_argument("--vmm-latency", action="store_true",
                    help="also time the driver's virtual-memory calls per 2 MiB chunk (the paper's mapping mechanism)")
    ap.add_argument("--prefill-append", type=int, default=0, metavar="N",
                    help="also time a multi-token append of N tokens per request and layer")
    return ap.parse_args()


DEFAULT_LAYERS = {"llama8b": 32, "mha13b": 2, "long70b": 4, "tiny": 4}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(the path needs no collective and nothing in it spans GPUs)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2506_15155_amd as E
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config]
    n_layers = args.layers or DEFAULT_LAYERS[args.config]
    K, Wm = args.steps, args.warmup
    B, Hq, Hkv, D, Tc = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.tokens_per_chunk
    rng = np.random.default_rng(cfg.seed)
    lens_final = W.draw_lengths(cfg, rng)                  # lengths after the LAST timed step
    grow = K + Wm + (0 if args.no_cpu_baseline else 1)
    lens0 = np.maximum(lens_final - grow, 1)               # lengths before the first step's append
    max_tokens = int(lens_final.max()) + Tc

    # one unified pool for all layers; 1/8 of it starts on the activation side (idle), so that
    # map-ahead can borrow from it when the KV side runs dry
    slots_now = [int(-(-int(l) // Tc)) for l in lens0]
    need = n_layers * sum(slots_now)
    n_chunks = int(need * 1.15) + 64
    if args.prefill_append:
        n_chunks += n_layers * B * -(-args.prefill_append // Tc)
    if args.migration:
        n_chunks += 512        # room for the chunks of two layers' parked requests to be resident at once
    owner = np.zeros(n_chunks, np.uint8)
    owner[rng.random(n_chunks) < 0.125] = 1
    kv_ids = np.flatnonzero(owner == 0).astype(np.int32)
    if args.placement == "shuffled":
        rng.shuffle(kv_ids)
    dev_bytes = n_chunks * cfg.chunk_bytes
    if args.pool_memory == "vmm":
        dev, dev_bytes = E.ellm_debug_vmm_buffer_create(cfg.chunk_bytes, n_chunks, cfg.seed, 0x7FC0)   # an address
    else:
        dev = torch.empty(dev_bytes, dtype=torch.uint8, device="cuda")
        dev.view(torch.int16).fill_(0x7FC0)                # NaN poison everywhere that is not KV
    n_host = 0
    host = None
    if args.migration:
        n_host = n_layers * sum(-(-(int(lens_final[b]) + 64) // Tc) for b in range(0, B, 4))
        host = torch.empty(n_host * cfg.chunk_bytes, dtype=torch.uint8, pin_memory=True)
    pool = E.ellm_pool_create(dev, host, cfg.chunk_bytes, Hq, Hkv, D,
                              n_layers * B * (2 if args.prefill_append else 1), -(-max_tokens // Tc), owner,
                              device_bytes=dev_bytes)
    if args.split:
        E.ellm_pool_set_split_tokens(pool, args.split)
    if args.waves_percent:
        E.ellm_debug_set_waves(pool, args.waves_percent)

    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed)
    n_oracle_layers = 0 if args.no_cpu_baseline else 1
    oracle_hist = []
    ids, pos = [], 0
    for l in range(n_layers):
        lid = []
        for b in range(B):
            t = E.ellm_tensor_create(pool, max_tokens)
            E.ellm_tensor_map_chunks(pool, t, 0, slots_now[b], kv_ids[pos:pos + slots_now[b]])
            pos += slots_now[b]
            lid.append(t)
        ids.append(np.array(lid, np.int32))
        tot = int(lens0.sum())
        k = torch.randn((tot, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        v = torch.randn((tot, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        E.ellm_kv_append(pool, ids[l], k, v, lens0.astype(np.int32))
        if l < n_oracle_layers:
            oracle_hist.append((k.view(torch.int16).cpu().numpy().view(np.uint16),
                                v.view(torch.int16).cpu().numpy().view(np.uint16)))
        torch.cuda.synchronize()
        del k, v
    k_new = [torch.randn((B, Hkv, D), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(n_layers)]
    v_new = [torch.randn((B, Hkv, D), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(n_layers)]
    q = [torch.randn((B, Hq, D), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(n_layers)]
    out = [torch.empty((B, Hq, D), device="cuda", dtype=torch.bfloat16) for _ in range(n_layers)]
    stream = torch.cuda.current_stream()

    lens = lens0.copy()

    # the timed loop calls the C ABI with arguments marshalled once, so the host stays ahead of the GPU
    import ctypes as C
    c_pool, c_stream = C.c_void_p(pool), C.c_void_p(stream.cuda_stream or None)
    c_ids = [a.ctypes.data_as(C.POINTER(C.c_int32)) for a in ids]
    c_k = [C.c_void_p(t.data_ptr()) for t in k_new]
    c_v = [C.c_void_p(t.data_ptr()) for t in v_new]
    c_q = [C.c_void_p(t.data_ptr()) for t in q]
    c_o = [C.c_void_p(t.data_ptr()) for t in out]
    c_scale = C.c_float(0.0)
    f_append, f_decode, f_fused = E.lib.ellm_kv_append, E.lib.ellm_decode_attention, E.lib.ellm_kv_append_decode
    fused = not args.separate_calls

    f_premap = E.lib.ellm_kv_premap_next
    c_inflate = C.c_uint32(E.ELLM_MAP_ALLOW_INFLATE)

    def map_ahead():
        # a3: requests whose next token opens a new chunk get one mapped (inflating if needed)
        if not (lens % Tc == 0).any():
            return
        for l in range(n_layers):
            if f_premap(c_pool, c_ids[l], B, c_inflate, None):
                raise E.EllmError(-1, E.ellm_last_error())

    def layer_call(l):
        if fused:
            rc = f_fused(c_pool, c_ids[l], B, c_k[l], c_v[l], c_q[l], c_o[l], c_scale, c_stream)
        else:
            rc = f_append(c_pool, c_ids[l], B, None, c_k[l], c_v[l], c_stream)
            rc |= f_decode(c_pool, c_ids[l], B, c_q[l], c_o[l], c_scale, c_stream)
        if rc:
            raise E.EllmError(rc, E.ellm_last_error())

    def step():
        map_ahead()
        for l in range(n_layers):
            layer_call(l)
        lens[:] += 1

    for _ in range(Wm):
        step()
    torch.cuda.synchronize()
    use_events = not args.no_kernel_events
    if use_events:
        # every 7th launch is timed (7 and the layer count share no factor, so every layer gets its turn):
        # an event pair costs about 3 us of stream time, 7 % of the step if it sat around every launch
        E.ellm_pool_profile_enable(pool, K * n_layers * 2)
        E.ellm_pool_profile_stride(pool, args.event_stride)
    n_split_now, S = E.ellm_decode_plan(pool, ids[0])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    kern_ms = E.ellm_pool_profile_collect(pool, K * n_layers * 2) if use_events else np.zeros(0, np.float32)
    if use_events:
        E.ellm_pool_profile_enable(pool, 0)

    # algorithmic bytes: lengths at the middle of the timed region
    lens_mid = lens - (K + 1) // 2
    n_items = int(np.sum(n_split_now))          # partial results per kv-head group, from the library's plan
    ab = W.algorithmic_bytes(cfg, lens_mid, n_items)
    step_bytes = ab["total"] * n_layers
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    # dominant kernel: the partial pass reads K/V, q and table entries and writes the partials; fused, it
    # also reads the new token's K/V rows and writes them into their chunks
    partial_bytes = ab["kv"] + ab["q_out"] // 2 + ab["table"] + ab["partials"] // 2 + (ab["append"] if fused else 0)
    roofline = None
    if use_events and len(kern_ms):
        avg = float(np.mean(kern_ms))
        ach = partial_bytes / (avg * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "decode_partial_kernel", "achieved": round(ach, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None,
                    "avg_launch_us": round(avg * 1e3, 2), "launches": int(len(kern_ms)),
                    "algorithmic_bytes_per_launch": int(partial_bytes)}

    if roofline is not None and not args.no_ceilings:
        roofline.update(read_ceilings(E, torch, pool, dev, dev_bytes, ids, partial_bytes, ab["kv"]))
        roofline["frac_of_measured_read_ceiling"] = round(ach / roofline["contiguous_read_GBps"], 4)
    if roofline is not None and args.config == "llama8b" and n_layers == 32 and not args.split:
        roofline["traffic"] = committed_traffic()

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, lens0, oracle_hist, ab, lens)

    mig = None
    if args.migration:
        mig = time_migration(E, torch, pool, ids, lens, Tc, cfg, B, n_layers, map_ahead, layer_call)
    turn = None
    if args.turnover:
        turn = time_turnover(E, torch, pool, ids, lens, cfg, n_layers, max_tokens)
    pre = None
    if args.prefill_append:
        pre = time_prefill_append(E, torch, pool, ids, lens, cfg, n_layers, args.prefill_append, max_tokens)

    res = {
        "metric": "decode-attention achieved HBM GB/s (% of peak) + tokens/s, chunk-backed KV, 1 GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "pct_of_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "tokens_per_s": round(B / (ms_per_step * 1e-3), 1),
        "tokens_per_s_per_layer": round(B * n_layers / (ms_per_step * 1e-3), 1),
        "config": {"workload": f"{args.config}: {Hq}q/{Hkv}kv heads, head_dim {D}, batch {B}, {n_layers} layers, "
                               f"lengths {cfg.length_dist} {cfg.len_lo}..{cfg.len_hi} (mean {float(lens_mid.mean()):.0f}), "
                               f"{cfg.chunk_bytes >> 10} KiB chunks "
                               + ("shuffled" if args.placement == "shuffled" else "in consecutive runs per tensor")
                               + f" in one pool of {n_chunks}"
                               + (" (each chunk a physical allocation of its own, driver-mapped)" if args.pool_memory == "vmm" else "")
                               + ", "
                               "step = per layer map-ahead + append 1 token/request + decode"
                               + (" (one fused call)" if fused else " (two calls)"),
                   "global_batch": B, "layers": n_layers, "split_tokens": int(S), "work_items_per_layer": n_items,
                   "algorithmic_bytes_per_step": int(step_bytes)},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if mig:
        res["migration"] = mig
    if pre:
        res["prefill_append"] = pre
    if turn:
        res["turnover"] = turn
    if args.vmm_latency:
        rc, us = E.ellm_debug_vmm_latency(cfg.chunk_bytes, 256, check=False)
        res["vmm_us_per_chunk"] = ({"create": round(us[0], 2), "map_and_set_access": round(us[1], 2), "unmap": round(us[2], 2),
                                    "release": round(us[3], 2), "chunks": 256} if rc == 0
                                   else {"error": E.ellm_last_error()})
    E.ellm_pool_destroy(pool)
    if args.pool_memory == "vmm":
        E.ellm_debug_vmm_buffer_destroy(dev)
    print(json.dumps(res))


def read_ceilings(E, torch, pool, dev, dev_bytes, ids, partial_bytes, kv_bytes):
    """What plain reads reach on this GPU, for scale: one contiguous read of as many bytes as the
    partial pass moves, and a read-only kernel that walks the same K/V tiles through the same chunk
    tables with the same cut into per-wave shares (no arithmetic, nothing written)."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")

    def timed(fn, n):
        fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    nb = min(int(partial_bytes), dev_bytes) // 16 * 16
    ms_c = timed(lambda i: E.ellm_debug_stream_read(dev, nb, sink), 40)
    ms_k = timed(lambda i: E.ellm_debug_kv_stream_read(pool, ids[i % len(ids)], sink), 4 * len(ids))
    # a plain copy of known size: the yardstick that scales the FETCH_SIZE / WRITE_SIZE counters
    src = torch.zeros(COPY_CALIBRATION_BYTES, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    timed(lambda i: E.ellm_debug_copy(dst, src, COPY_CALIBRATION_BYTES), 3)
    return {"contiguous_read_GBps": round(nb / ms_c / 1e6, 1), "kv_pattern_read_GBps": round(kv_bytes / ms_k / 1e6, 1)}


def committed_traffic():
    """HBM bytes per launch of the partial pass from the committed counter runs (rocprofv3 --pmc
    FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for a copy of known
    size). The summary file states the commands; None when it is absent."""
    path = os.path.join(ROOT, "profiles", "decode_partial_llama8b_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1].split()[0]))
    except OSError:
        pass
    return None


def cpu_baseline(cfg, lens0, oracle_hist, ab, lens_now, budget_s=15.0):
    """The oracle, as it stands, on the host cores: one layer of the same workload, all requests.
    Loading the history is setup; the timed part is consecutive append + decode steps (new K/V/q
    every step) until about `budget_s` seconds of oracle work are done."""
    import workloads as W
    from oracle.model import OraclePool
    B, Tc = cfg.batch, cfg.tokens_per_chunk
    max_steps = 400
    slots = [int(-(-(int(l) + max_steps) // Tc)) for l in lens0]
    n_chunks = sum(slots)
    orc = OraclePool(n_chunks, cfg.chunk_bytes, 0, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, B,
                     max(slots), None, False)
    rng = np.random.default_rng(cfg.seed + 1000)
    perm = rng.permutation(n_chunks).astype(np.int32)
    ids, pos = [], 0
    for b in range(B):
        rc, t = orc.tensor_create(max(slots) * Tc)
        assert rc == 0 and orc.map_chunks(t, 0, slots[b], perm[pos:pos + slots[b]]) == 0
        pos += slots[b]
        ids.append(t)
    kh, vh = oracle_hist[0]
    assert orc.append(ids, kh, vh, lens0.astype(np.int32)) == 0
    cores = os.cpu_count() or 1
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    spent, nbytes, n_steps, lens = 0.0, 0, 0, lens0.copy()
    while spent < budget_s and n_steps < max_steps:
        k1 = W.normal_bf16(rng, (B, cfg.n_kv_heads, cfg.head_dim))
        v1 = W.normal_bf16(rng, (B, cfg.n_kv_heads, cfg.head_dim))
        q1 = W.normal_bf16(rng, (B, cfg.n_q_heads, cfg.head_dim))
        t0 = time.perf_counter()
        rc = orc.append(ids, k1, v1)
        rc2, _ = orc.decode(ids, q1, threads=cores)
        spent += time.perf_counter() - t0
        assert rc == 0 and rc2 == 0
        lens += 1
        n_steps += 1
        nbytes += W.algorithmic_bytes(cfg, lens, 0)["total"]
    orc.close()
    return {"value": round(nbytes / spent / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"1 of the layers, all {B} requests, {n_steps} consecutive append + decode steps "
                      f"({int(lens.sum())} cached tokens at the end), fp64 C oracle with pthreads",
            "seconds": round(spent, 3), "tokens_per_s_per_layer": round(B * n_steps / spent, 2)}


def time_migration(E, torch, pool, ids, lens, Tc, cfg, B, n_layers, map_ahead, layer_call):
    """Two cases: every 4th request parked (the elastic configuration; the copies take far longer than
    the step), and one request of median length parked (copies of the order of the step)."""
    order = np.argsort(lens)
    return {"quarter_of_requests": _time_migration(E, torch, pool, ids, lens, Tc, cfg, n_layers, map_ahead, layer_call,
                                                   list(range(0, B, 4)), 3),
            "one_median_request": _time_migration(E, torch, pool, ids, lens, Tc, cfg, n_layers, map_ahead, layer_call,
                                                  [int(order[B // 2])], 10)}


def _time_migration(E, torch, pool, ids, lens, Tc, cfg, n_layers, map_ahead, layer_call, sel, steps):
    """The elastic step over all layers with every 4th request parked in pinned host memory between
    steps: (a) no migration, (b) fetch everything, wait, run the step, offload everything, (c) layer by
    layer: the fetch of layer l+1 is issued before layer l's attention and the offload of layer l
    right after it, so the copies run on the side stream under the kernels."""

    def slots(b, extra=0):
        return int(-(-(int(lens[b]) + extra) // Tc))

    def offload_layer(l, extra=0):
        for b in sel:
            E.ellm_chunk_deflate_to_host(pool, int(ids[l][b]), 0, slots(b, extra))

    def fetch_layer(l):
        for b in sel:
            E.ellm_chunk_inflate_from_host(pool, int(ids[l][b]), 0, slots(b))

    def sync():
        E.ellm_pool_sync(pool)
        torch.cuda.synchronize()

    def timed(fn):
        sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        sync()
        return (time.perf_counter() - t0) * 1e3 / steps

    def plain():
        map_ahead()
        for l in range(n_layers):
            layer_call(l)
        lens[:] += 1

    def copies_only():
        for l in range(n_layers):
            fetch_layer(l)
        for l in range(n_layers):
            offload_layer(l)

    def blocking():
        for l in range(n_layers):
            fetch_layer(l)
        E.ellm_pool_sync(pool)
        map_ahead()
        for l in range(n_layers):
            layer_call(l)
        torch.cuda.synchronize()
        for l in range(n_layers):
            offload_layer(l, 1)
        lens[:] += 1

    def layerwise():
        map_ahead()
        fetch_layer(0)
        for l in range(n_layers):
            if l + 1 < n_layers:
                fetch_layer(l + 1)
            layer_call(l)
            offload_layer(l, 1)
        lens[:] += 1

    t_plain = timed(plain)
    for l in range(n_layers):          # park the selected requests
        offload_layer(l)
    sync()
    nbytes = sum(slots(b) for b in sel) * cfg.chunk_bytes * n_layers
    t_copy = timed(copies_only)
    t_block = timed(blocking)
    t_layer = timed(layerwise)
    for l in range(n_layers):          # leave everything resident
        fetch_layer(l)
    sync()
    return {"parked_requests": len(sel), "bytes_each_way_per_step": int(nbytes),
            "ms_step_no_migration": round(t_plain, 3), "ms_copies_only": round(t_copy, 3),
            "ms_step_fetch_all_then_compute": round(t_block, 3), "ms_step_layerwise": round(t_layer, 3),
            "pcie_GBps_both_ways_avg": round(2 * nbytes / (t_copy * 1e-3) / 1e9, 2),
            "ms_hidden_by_layerwise": round(t_block - t_layer, 3)}


def time_turnover(E, torch, pool, ids, lens, cfg, n_layers, max_tokens, rounds=20):
    """Host cost of replacing a finished request by a new one of the same prompt length in every layer:
    (a) release + acquire, where the best-fitting available tensor is taken with its mapping intact and
    no table entry changes; (b) destroy + create + map, where every slot is mapped again and the device
    table has to be patched. Microseconds per request and layer; the tensors end up as they started."""
    B, Tc = cfg.batch, cfg.tokens_per_chunk
    order = np.argsort(lens)
    pick = [int(order[B // 2]), int(order[3 * B // 4]), int(order[B // 4])]
    torch.cuda.synchronize()
    t_reuse = t_remap = 0.0
    n_ops = 0
    for _ in range(rounds):
        for b in pick:
            need = int(lens[b])
            t0 = time.perf_counter()
            for l in range(n_layers):
                E.ellm_tensor_release(pool, int(ids[l][b]))
            for l in range(n_layers):
                t = E.ellm_tensor_acquire(pool, need, max_tokens)
                ids[l][b] = t
            t1 = time.perf_counter()
            for l in range(n_layers):
                E.ellm_tensor_destroy(pool, int(ids[l][b]))
            for l in range(n_layers):
                t = E.ellm_tensor_create(pool, max_tokens)
                E.ellm_tensor_map_chunks(pool, t, 0, -(-need // Tc), None, E.ELLM_MAP_ALLOW_INFLATE)
                ids[l][b] = t
            t2 = time.perf_counter()
            t_reuse += t1 - t0
            t_remap += t2 - t1
            n_ops += n_layers
    # the tensors are empty now: give them their length back (contents do not matter any more)
    kd = torch.zeros((int(lens.max()), cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    for b in pick:
        for l in range(n_layers):
            E.ellm_kv_append(pool, [int(ids[l][b])], kd, kd, [int(lens[b])])
    torch.cuda.synchronize()
    return {"us_release_plus_best_fit_acquire": round(t_reuse / n_ops * 1e6, 2),
            "us_destroy_create_map": round(t_remap / n_ops * 1e6, 2),
            "slots_per_request": [int(-(-int(lens[b]) // Tc)) for b in pick],
            "note": "host time per request and layer through the Python binding; the second path also leaves one "
                    "table entry per slot to be patched on the device by the next call"}


def time_prefill_append(E, torch, pool, ids, lens, cfg, n_layers, n_tok, max_tokens):
    """Multi-token append (the prefill-side write): n_tok tokens per request into fresh tensors of every
    layer; GB/s counts the new K/V rows read and written."""
    B, Tc = cfg.batch, cfg.tokens_per_chunk
    n_tok = min(n_tok, max_tokens)
    need = -(-n_tok // Tc)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed + 9)
    k = torch.randn((B * n_tok, cfg.n_kv_heads, cfg.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    v = torch.randn((B * n_tok, cfg.n_kv_heads, cfg.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    counts = np.full(B, n_tok, np.int32)
    times = []
    for rep in range(3):
        fresh = []
        try:
            for l in range(n_layers):
                row = []
                for b in range(B):
                    t = E.ellm_tensor_create(pool, max_tokens)
                    row.append(t)
                    E.ellm_tensor_map_chunks(pool, t, 0, need, None, E.ELLM_MAP_ALLOW_INFLATE)
                fresh.append(np.array(row, np.int32))
        except E.EllmError as e:
            for row in fresh:
                for t in row:
                    E.ellm_tensor_destroy(pool, int(t))
            return {"skipped": f"pool has no room for the extra tensors ({e})"}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for l in range(n_layers):
            E.ellm_kv_append(pool, fresh[l], k, v, counts)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        for row in fresh:
            for t in row:
                E.ellm_tensor_destroy(pool, int(t))
    nbytes = 2 * 2 * B * n_tok * cfg.n_kv_heads * cfg.head_dim * 2 * n_layers
    best = min(times)
    return {"tokens_per_request": n_tok, "ms_all_layers": round(best * 1e3, 3), "GBps": round(nbytes / best / 1e9, 1)}


if __name__ == "__main__":
    main()
