"""Benchmark: decode attention + KV append over chunk-backed KV on one MI355X.

Headline workload (default): the Llama-3-8B-shaped configuration — 32 q / 8 kv heads, head_dim 128,
bf16, batch 64, context lengths lognormal (median 1k, clipped 64..8k), 2 MiB chunks shuffled in one
unified pool — for all 32 layers of such a model: every (layer, request) is a virtual KV tensor of
its own, so one step streams 32 different layers' K/V (about 12 GB) and no cache level can serve the
reads. One step = for every layer: map a chunk ahead for requests about to cross a chunk boundary,
append one token per request, decode-attend over the whole context.

Prints ONE JSON line. `value` is the headline workload's whole-step GB/s of algorithmic bytes; `roofline`
the attention kernel's HIP-event time per launch against the 8 TB/s HBM peak; `cpu_baseline` the fp64
CPU oracle timed on the host cores; `parity` the last timed step's output of one layer against the
oracle on the same bits. With the default workload the line also carries, under `workloads`, the
13B-shaped MHA layer and the 70B-shaped long-context layer measured the same way, the elastic step
(chunks handed over from the activation side, a quarter of the requests offloaded to pinned host and
fetched back) and the same model in a driver-mapped pool (the paper's own mapping mechanism); then
every workload runs in a process of its own, one after the other, and this one only merges their lines.
"""
from __future__ import annotations

import argparse
import ctypes as C
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
DEFAULT_LAYERS = {"llama8b": 32, "mha13b": 2, "long70b": 4, "tiny": 4}
METRIC = "decode-attention achieved HBM GB/s (% of peak) + tokens/s, chunk-backed KV, 1 GPU"


LEGS = ["elastic", "driver_mapped", "long70b", "mha13b"]      # the other workloads of the default run


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="llama8b", choices=["llama8b", "mha13b", "long70b", "tiny"])
    ap.add_argument("--layers", type=int, default=0, help="0 = the layer count used for the shape")
    ap.add_argument("--extras", dest="extras", action="store_true", default=None,
                    help="also measure the other workloads (default with --config llama8b)")
    ap.add_argument("--no-extras", dest="extras", action="store_false")
    ap.add_argument("--split", type=int, default=0, help="override tokens per wave (0 = automatic)")
    ap.add_argument("--waves-percent", type=int, default=0,
                    help="waves per decode launch as a percentage of the library's choice, one wave per SIMD (0 = leave it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--event-stride", type=int, default=0,
                    help="time every n-th attention launch with HIP events (0 = 13 for the 8B-shaped workload, whose "
                         "launches are short, 1 for the others)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured read ceilings")
    ap.add_argument("--separate-calls", action="store_true",
                    help="ellm_kv_append then ellm_decode_attention instead of the fused ellm_kv_append_decode")
    ap.add_argument("--pool", default="plain", choices=["plain", "driver-mapped", "driver-mapped-table-kernels"],
                    help="driver-mapped: ELLM_POOL_DRIVER_MAPPED, kernels read each tensor's own address range; "
                         "-table-kernels: the same pool read through the software table")
    ap.add_argument("--pool-memory", default="malloc", choices=["malloc", "vmm"],
                    help="vmm: a plain pool over a buffer whose 2 MiB pieces are physical allocations of their own")
    ap.add_argument("--placement", default="shuffled", choices=["shuffled", "contiguous"])
    ap.add_argument("--turnover", action="store_true", help="also time request turnover on the host")
    ap.add_argument("--vmm-latency", action="store_true", help="also time the driver's virtual-memory calls per chunk")
    ap.add_argument("--prefill-append", type=int, default=0, metavar="N",
                    help="also time a multi-token append of N tokens per request and layer")
    ap.add_argument("--preheat", type=float, default=0.0, metavar="S",
                    help="read at full rate (decode calls, no append) for S seconds before the warm-up steps")
    ap.add_argument("--leg", default=None, choices=LEGS,
                    help="measure only this one of the other workloads, in this process, and print its figures")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------------
class Workload:
    """One configuration's layers in one unified pool, loaded and ready to step."""

    def __init__(self, E, torch, W, name, n_layers, grow, pool_kind="plain", pool_memory="malloc", placement="shuffled",
                 host_for_quarter=False, extra_chunks=0, extra_tensors=0, keep_hist_for=(), split=0, waves_percent=0):
        self.E, self.torch, self.W = E, torch, W
        self.name, self.cfg, self.n_layers = name, W.CONFIGS[name], n_layers
        cfg = self.cfg
        B, Hq, Hkv, D, Tc = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.tokens_per_chunk
        rng = np.random.default_rng(cfg.seed)
        # the configuration's seeded lengths are the lengths half-way through the steps this object will
        # run, so that the measured workload does not depend on how many steps are timed
        mid = W.draw_lengths(cfg, rng)
        self.lens0 = np.maximum(mid - (grow + 1) // 2, 1)      # lengths before the first step's append
        self.lens_final = self.lens0 + grow
        self.max_tokens = int(self.lens_final.max()) + Tc
        slots_now = [int(-(-int(l) // Tc)) for l in self.lens0]
        need = n_layers * sum(slots_now)
        self.n_chunks = int(need * 1.15) + 64 + extra_chunks
        # 1/8 of the pool starts on the activation side (idle), so that map-ahead can borrow from it
        owner = np.zeros(self.n_chunks, np.uint8)
        owner[rng.random(self.n_chunks) < 0.125] = 1
        self.owner0 = owner
        kv_ids = np.flatnonzero(owner == 0).astype(np.int32)
        if placement == "shuffled":
            rng.shuffle(kv_ids)
        self.dev_bytes = self.n_chunks * cfg.chunk_bytes
        self.vmm_buffer = None
        self.pool_kind = pool_kind
        self.host = None
        n_host = 0
        if host_for_quarter:
            n_host = n_layers * sum(-(-(int(self.lens_final[b]) + 64) // Tc) for b in range(0, B, 4))
            self.host = torch.empty(n_host * cfg.chunk_bytes, dtype=torch.uint8, pin_memory=True)
        mt = n_layers * B + extra_tensors
        if pool_kind != "plain":
            self.dev = None
            self.pool = E.ellm_pool_create(None, self.host, cfg.chunk_bytes, Hq, Hkv, D, mt, -(-self.max_tokens // Tc), owner,
                                           flags=E.ELLM_POOL_DRIVER_MAPPED, device_bytes=self.dev_bytes)
            self.base = E.ellm_pool_get_device_base(self.pool)
            fill = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
            fill.view(torch.int16).fill_(0x7FC0)
            for off in range(0, self.dev_bytes, fill.numel()):
                E.ellm_debug_copy(self.base + off, fill, min(fill.numel(), self.dev_bytes - off))
            torch.cuda.synchronize()
            del fill
            if pool_kind == "driver-mapped-table-kernels":
                E.ellm_debug_set_table_kernels(self.pool, 1)
        else:
            if pool_memory == "vmm":
                self.dev, self.dev_bytes = E.ellm_debug_vmm_buffer_create(cfg.chunk_bytes, self.n_chunks, cfg.seed, 0x7FC0)
                self.vmm_buffer = self.dev
            else:
                self.dev = torch.empty(self.dev_bytes, dtype=torch.uint8, device="cuda")
                self.dev.view(torch.int16).fill_(0x7FC0)       # NaN poison everywhere that is not KV
            self.pool = E.ellm_pool_create(self.dev, self.host, cfg.chunk_bytes, Hq, Hkv, D, mt, -(-self.max_tokens // Tc),
                                           owner, device_bytes=self.dev_bytes)
            self.base = self.dev
        if split:
            E.ellm_pool_set_split_tokens(self.pool, split)
        if waves_percent:
            E.ellm_debug_set_waves(self.pool, waves_percent)

        gen = torch.Generator(device="cuda")
        gen.manual_seed(cfg.seed)
        self.hist = {}                 # layer -> (K bits, V bits) on the host, for the layers in keep_hist_for
        self.hist_rows = None          # which requests' rows were kept (None = all)
        self.ids, pos = [], 0
        t_setup_maps = time.perf_counter()
        for l in range(n_layers):
            lid = []
            for b in range(B):
                t = E.ellm_tensor_create(self.pool, self.max_tokens)
                E.ellm_tensor_map_chunks(self.pool, t, 0, slots_now[b], kv_ids[pos:pos + slots_now[b]])
                pos += slots_now[b]
                lid.append(t)
            self.ids.append(np.array(lid, np.int32))
        self.setup_map_s = time.perf_counter() - t_setup_maps
        self.setup_slots = pos
        for l in range(n_layers):
            tot = int(self.lens0.sum())
            k = torch.randn((tot, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            v = torch.randn((tot, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            E.ellm_kv_append(self.pool, self.ids[l], k, v, self.lens0.astype(np.int32))
            if l in keep_hist_for:
                self.hist[l] = (k, v)          # converted to host bits on demand (sampled rows only for big shapes)
            torch.cuda.synchronize()
            if l not in keep_hist_for:
                del k, v
        self.k_new = [torch.randn((B, Hkv, D), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(n_layers)]
        self.v_new = [torch.randn((B, Hkv, D), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(n_layers)]
        self.q = [torch.randn((B, Hq, D), generator=gen, device="cuda").to(torch.bfloat16) for _ in range(n_layers)]
        self.out = [torch.empty((B, Hq, D), device="cuda", dtype=torch.bfloat16) for _ in range(n_layers)]
        self.stream = torch.cuda.current_stream()
        self.lens = self.lens0.copy()
        self.steps_done = 0
        self.mapped_slots = np.array(slots_now, np.int64)
        self.map_lookahead = None       # a number: slots are mapped one by one, that many steps before their first
                                        # write (0: in the step itself); None: by the library's pre-mapping call

        # the timed loop calls the C ABI with arguments marshalled once, so the host stays ahead of the GPU
        self.c_pool, self.c_stream = C.c_void_p(self.pool), C.c_void_p(self.stream.cuda_stream or None)
        self.c_ids = [a.ctypes.data_as(C.POINTER(C.c_int32)) for a in self.ids]
        self.c_k = [C.c_void_p(t.data_ptr()) for t in self.k_new]
        self.c_v = [C.c_void_p(t.data_ptr()) for t in self.v_new]
        self.c_q = [C.c_void_p(t.data_ptr()) for t in self.q]
        self.c_o = [C.c_void_p(t.data_ptr()) for t in self.out]
        self.c_scale = C.c_float(0.0)
        self.c_inflate = C.c_uint32(E.ELLM_MAP_ALLOW_INFLATE)
        self.fused = True

    def map_ahead(self):
        E, B, Tc = self.E, self.cfg.batch, self.cfg.tokens_per_chunk
        if self.map_lookahead is not None:
            # a driver-mapped pool is told some steps early (the paper maps ahead of time, Sec. 3.1): the
            # pool's mapper thread then has made the driver calls by the time the slot is written
            ahead = self.map_lookahead + 1          # tokens: this step's and those of the steps after it
            if not ((self.lens + ahead - 1) // Tc >= self.mapped_slots).any():
                return
            for l in range(self.n_layers):
                if E.lib.ellm_kv_premap_ahead(self.c_pool, self.c_ids[l], B, C.c_int64(ahead), self.c_inflate, None):
                    raise E.EllmError(-1, E.ellm_last_error())
            self.mapped_slots = np.maximum(self.mapped_slots, (self.lens + ahead - 1) // Tc + 1)
            return
        # requests whose next token opens a new chunk get one mapped (inflating if needed)
        if not (self.lens % Tc == 0).any():
            return
        for l in range(self.n_layers):
            if E.lib.ellm_kv_premap_next(self.c_pool, self.c_ids[l], B, self.c_inflate, None):
                raise E.EllmError(-1, E.ellm_last_error())

    def layer_call(self, l):
        E, B = self.E, self.cfg.batch
        if self.fused:
            rc = E.lib.ellm_kv_append_decode(self.c_pool, self.c_ids[l], B, self.c_k[l], self.c_v[l], self.c_q[l], self.c_o[l],
                                             self.c_scale, self.c_stream)
        else:
            rc = E.lib.ellm_kv_append(self.c_pool, self.c_ids[l], B, None, self.c_k[l], self.c_v[l], self.c_stream)
            rc |= E.lib.ellm_decode_attention(self.c_pool, self.c_ids[l], B, self.c_q[l], self.c_o[l], self.c_scale, self.c_stream)
        if rc:
            raise E.EllmError(rc, E.ellm_last_error())

    def step(self):
        self.map_ahead()
        for l in range(self.n_layers):
            self.layer_call(l)
        self.lens[:] += 1
        self.steps_done += 1

    def n_split_items(self):
        """Partial results per kv head that a launch writes to the workspace and the combine pass reads:
        requests that lie inside one wave's share have none."""
        n_split, S = self.E.ellm_decode_plan(self.pool, self.ids[0])
        return int(n_split[n_split > 1].sum()), int(S), int((n_split > 1).sum())

    def close(self):
        self.torch.cuda.synchronize()
        self.E.ellm_pool_destroy(self.pool)
        if self.vmm_buffer is not None:
            self.E.ellm_debug_vmm_buffer_destroy(self.vmm_buffer)
        self.dev = None
        self.host = None


def measure(wl, K, Wm, event_stride=0, use_events=True, preheat_s=0.0):
    """Wm untimed steps, then K timed steps between device synchronisations: wall clock for the mean
    (inputs resident in HBM), one stream event per step for the spread, the library's own event pairs
    around every event_stride-th attention kernel for the roofline. preheat_s: before all that, the
    layers' decode calls (no append: the lengths stay) are repeated for that many seconds, so that the
    timed steps run on a GPU that has been reading at full rate for a while."""
    E, torch, W, cfg = wl.E, wl.torch, wl.W, wl.cfg
    if not event_stride:
        event_stride = 13 if wl.name in ("llama8b", "tiny") else 1
    if preheat_s > 0:
        t_end = time.perf_counter() + preheat_s
        while time.perf_counter() < t_end:
            for _ in range(8):
                for l in range(wl.n_layers):
                    rc = E.lib.ellm_decode_attention(wl.c_pool, wl.c_ids[l], cfg.batch, wl.c_q[l], wl.c_o[l], wl.c_scale, wl.c_stream)
                    if rc:
                        raise E.EllmError(rc, E.ellm_last_error())
            torch.cuda.synchronize()
    for _ in range(Wm):
        wl.step()
    torch.cuda.synchronize()
    if use_events:
        # 13 and the layer count share no factor, so every layer gets its turn; an event pair costs about 3 us
        # of stream time, 7 % of the 8B-shaped step if it sat around every launch
        E.ellm_pool_profile_enable(wl.pool, K * wl.n_layers * 2)
        E.ellm_pool_profile_stride(wl.pool, event_stride)
    n_items, S, n_split_req = wl.n_split_items()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(K):
        wl.step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    per_step = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(K)])
    kern_ms = E.ellm_pool_profile_collect(wl.pool, K * wl.n_layers * 2) if use_events else np.zeros(0, np.float32)
    if use_events:
        E.ellm_pool_profile_enable(wl.pool, 0)

    lens_mid = wl.lens - (K + 1) // 2                      # algorithmic bytes: lengths at the middle of the timed region
    ab = W.algorithmic_bytes(cfg, lens_mid, n_items)
    step_bytes = ab["total"] * wl.n_layers
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    # the attention kernel reads K/V, q and table entries, writes the partials of the split requests and the
    # output rows of the others; fused, it also reads the new token's K/V rows and writes them into their chunks
    B, Hq, D = cfg.batch, cfg.n_q_heads, cfg.head_dim
    direct_out = (B - n_split_req) * Hq * D * 2
    partial_bytes = ab["kv"] + ab["q_out"] // 2 + ab["table"] + ab["partials"] // 2 + direct_out + (ab["append"] if wl.fused else 0)
    res = {
        "value": round(value, 1), "unit": "GB/s", "pct_of_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "ms_per_step": round(ms_per_step, 4), "steps": K, "warmup": Wm, "layers": wl.n_layers,
        "ms_per_step_median": round(float(np.median(per_step)), 4),
        "ms_per_step_p10": round(float(np.percentile(per_step, 10)), 4),
        "ms_per_step_p90": round(float(np.percentile(per_step, 90)), 4),
        "us_per_layer": round(ms_per_step * 1e3 / wl.n_layers, 2),
        "tokens_per_s": round(B / (ms_per_step * 1e-3), 1),
        "tokens_per_s_per_layer": round(B * wl.n_layers / (ms_per_step * 1e-3), 1),
        # the partial results are this implementation's own scratch traffic, not bytes the method has to move:
        "value_without_partials": round((step_bytes - ab["partials"] * wl.n_layers) / (ms_per_step * 1e-3) / 1e9, 1),
        "value_kv_only": round(ab["kv"] * wl.n_layers / (ms_per_step * 1e-3) / 1e9, 1),
        "mean_context": round(float(lens_mid.mean()), 1), "split_tokens": S,
        "partials_per_kv_head": n_items, "requests_finished_by_the_attention_kernel": B - n_split_req,
        "algorithmic_bytes_per_step": int(step_bytes),
    }
    roofline = None
    if use_events and len(kern_ms):
        avg = float(np.mean(kern_ms))
        ach = partial_bytes / (avg * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "decode_partial_kernel", "achieved": round(ach, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None,
                    "avg_launch_us": round(avg * 1e3, 2), "median_launch_us": round(float(np.median(kern_ms)) * 1e3, 2),
                    "launches": int(len(kern_ms)), "algorithmic_bytes_per_launch": int(partial_bytes)}
    res["roofline"] = roofline
    return res, ab, partial_bytes


def read_ceilings(wl, partial_bytes, kv_bytes):
    """What plain reads reach on this GPU, for scale: one contiguous read of as many bytes as the
    attention kernel moves, and a read-only kernel that walks the same K/V tiles through the same chunk
    tables with the same cut into per-wave shares (no arithmetic, nothing written)."""
    E, torch = wl.E, wl.torch
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

    nb = min(int(partial_bytes), wl.dev_bytes) // 16 * 16
    ms_c = timed(lambda i: E.ellm_debug_stream_read(wl.base, nb, sink), 40)
    ms_k = timed(lambda i: E.ellm_debug_kv_stream_read(wl.pool, wl.ids[i % len(wl.ids)], sink), 4 * len(wl.ids))
    # a plain copy of known size: the yardstick that scales the FETCH_SIZE / WRITE_SIZE counters
    src = torch.zeros(COPY_CALIBRATION_BYTES, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    timed(lambda i: E.ellm_debug_copy(dst, src, COPY_CALIBRATION_BYTES), 3)
    return {"contiguous_read_GBps": round(nb / ms_c / 1e6, 1), "kv_pattern_read_GBps": round(kv_bytes / ms_k / 1e6, 1)}


def committed_traffic(name):
    """HBM bytes per launch of the attention kernel from the committed counter runs (rocprofv3 --pmc
    FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for a copy of known size):
    separate runs of this program, not this one. Returns (bytes per launch, text naming the source)."""
    path = os.path.join(ROOT, "profiles", f"decode_partial_{name}_pmc.txt")
    got = {}
    try:
        for line in open(path):
            for key in ("traffic_bytes_per_launch", "algorithmic_bytes_per_launch", "traffic_over_algorithmic"):
                if line.startswith(key + ":"):
                    got[key] = float(line.split(":", 1)[1].split()[0])
    except OSError:
        return None, None
    if "traffic_bytes_per_launch" not in got:
        return None, None
    src = (f"profiles/decode_partial_{name}_pmc.txt: separate rocprofv3 --pmc runs of this program, not measured in this run"
           + (f"; algorithmic bytes per launch there {int(got['algorithmic_bytes_per_launch'])}" if "algorithmic_bytes_per_launch" in got else "")
           + (f", traffic / algorithmic {got['traffic_over_algorithmic']:.4f}" if "traffic_over_algorithmic" in got else ""))
    return int(got["traffic_bytes_per_launch"]), src


# ------------------------------------------------------------------------------------------------------
def host_bits(t):
    return t.view(wl_torch().int16).cpu().numpy().view(np.uint16)


def wl_torch():
    import torch
    return torch


def oracle_for_layer(wl, layer, sample):
    """The oracle's pool with the same logical KV as layer `layer` of the workload holds now, for the
    requests in `sample`: the seeded history plus one copy of the layer's new row per step done."""
    from oracle.model import OraclePool
    cfg, W = wl.cfg, wl.W
    Tc = cfg.tokens_per_chunk
    kh, vh = wl.hist[layer]
    starts = np.concatenate([[0], np.cumsum(wl.lens0)]).astype(np.int64)
    room = 400                                             # steps the baseline leg may add on top
    slots = [int(-(-(int(wl.lens[b]) + room) // Tc)) for b in sample]
    n_chunks = sum(slots)
    orc = OraclePool(n_chunks, cfg.chunk_bytes, 0, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, len(sample), max(slots),
                     None, False)
    rng = np.random.default_rng(cfg.seed + 1000)
    perm = rng.permutation(n_chunks).astype(np.int32)
    ids, pos = [], 0
    kn, vn = host_bits(wl.k_new[layer]), host_bits(wl.v_new[layer])
    for i, b in enumerate(sample):
        rc, t = orc.tensor_create(max(slots) * Tc)
        assert rc == 0 and orc.map_chunks(t, 0, slots[i], perm[pos:pos + slots[i]]) == 0
        pos += slots[i]
        ids.append(t)
        kb = host_bits(kh[starts[b]:starts[b + 1]])
        vb = host_bits(vh[starts[b]:starts[b + 1]])
        assert orc.append([t], kb, vb, [int(wl.lens0[b])]) == 0
        if wl.steps_done:
            rep_k = np.broadcast_to(kn[b], (wl.steps_done,) + kn[b].shape).copy()
            rep_v = np.broadcast_to(vn[b], (wl.steps_done,) + vn[b].shape).copy()
            assert orc.append([t], rep_k, rep_v, [wl.steps_done]) == 0
    return orc, ids


def parity_check(wl, layer, sample, threads):
    """The output the last step left for `layer` against the oracle's fp64 result on the same K/V/q bits."""
    orc, ids = oracle_for_layer(wl, layer, sample)
    qb = host_bits(wl.q[layer])[sample]
    rc, ref = orc.decode(ids, qb, threads=threads)
    assert rc == 0
    got = wl.W.f32_from_bf16_bits(host_bits(wl.out[layer])[sample]).astype(np.float64)
    err = np.abs(got - ref)
    res = {"layer": layer, "requests": len(sample), "of": wl.cfg.batch, "cached_tokens": int(sum(int(wl.lens[b]) for b in sample)),
           "max_abs": float(f"{err.max():.3e}"), "mean_abs": float(f"{err.mean():.3e}"),
           "finite": bool(np.isfinite(got).all()), "within_tolerance": bool(np.isfinite(got).all() and err.max() <= 2e-2 and err.mean() <= 2e-3),
           "tolerance": {"max_abs": 2e-2, "mean_abs": 2e-3}, "reference": "fp64 CPU oracle on the same bits"}
    return res, orc, ids


def cpu_baseline(wl, orc, ids, threads, budget_s=15.0):
    """The oracle, as it stands, on the host cores: one layer of the same workload, all requests,
    consecutive append + decode steps (new K/V/q every step) until about `budget_s` seconds are done."""
    cfg, W = wl.cfg, wl.W
    B = cfg.batch
    rng = np.random.default_rng(cfg.seed + 2000)
    spent, nbytes, n_steps, lens = 0.0, 0, 0, wl.lens.copy()
    while spent < budget_s and n_steps < 390:
        k1 = W.normal_bf16(rng, (B, cfg.n_kv_heads, cfg.head_dim))
        v1 = W.normal_bf16(rng, (B, cfg.n_kv_heads, cfg.head_dim))
        q1 = W.normal_bf16(rng, (B, cfg.n_q_heads, cfg.head_dim))
        t0 = time.perf_counter()
        rc = orc.append(ids, k1, v1)
        rc2, _ = orc.decode(ids, q1, threads=threads)
        spent += time.perf_counter() - t0
        assert rc == 0 and rc2 == 0
        lens += 1
        n_steps += 1
        nbytes += W.algorithmic_bytes(cfg, lens, 0)["total"]
    return {"value": round(nbytes / spent / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"1 of the layers, all {B} requests, {n_steps} consecutive append + decode steps "
                      f"({int(lens.sum())} cached tokens at the end), fp64 C oracle with pthreads",
            "seconds": round(spent, 3), "tokens_per_s_per_layer": round(B * n_steps / spent, 2)}


def host_threads():
    cores = os.cpu_count() or 1
    return min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))


# ------------------------------------------------------------------------------------------------------
def sub_workload(E, torch, W, name, K, Wm, args, n_sample):
    """A further configuration measured like the headline one, with the oracle check on sampled requests."""
    wl = Workload(E, torch, W, name, DEFAULT_LAYERS[name], K + Wm, keep_hist_for=(0,))
    res, ab, partial_bytes = measure(wl, K, Wm, args.event_stride)
    if res["roofline"] is not None and not args.no_ceilings:
        res["roofline"].update(read_ceilings(wl, partial_bytes, ab["kv"]))
        res["roofline"]["frac_of_measured_read_ceiling"] = round(res["roofline"]["achieved"] / res["roofline"]["contiguous_read_GBps"], 4)
    if res["roofline"] is not None:
        res["roofline"]["traffic"], src = committed_traffic(name)
        if src:
            res["roofline"]["traffic_source"] = src
    order = np.argsort(wl.lens, kind="stable")
    ranks = np.unique(np.rint(np.linspace(0, wl.cfg.batch - 1, n_sample)).astype(int))
    sample = sorted(int(order[r]) for r in ranks)          # shortest, longest and evenly spaced ranks between
    par, orc, _ = parity_check(wl, 0, sample, host_threads())
    orc.close()
    res["parity"] = par
    cfg = wl.cfg
    res["workload"] = (f"{name}: {cfg.n_q_heads}q/{cfg.n_kv_heads}kv heads, head_dim {cfg.head_dim}, batch {cfg.batch}, "
                       f"{wl.n_layers} layers in one pool of {wl.n_chunks} chunks, lengths {cfg.length_dist} "
                       f"{cfg.len_lo}..{cfg.len_hi}")
    wl.close()
    del wl
    torch.cuda.empty_cache()
    return res


def elastic_step(E, torch, W, args, steps=3):
    """The elastic configuration on the headline shapes: before each step a share of the idle activation
    chunks is handed to the KV side, every 4th request is offloaded to pinned host memory and fetched back
    into whatever chunks the pool picks, then all layers append and decode. Three numbers per step: the
    attention kernel's GB/s, the copy rate in each direction, the step's wall time (copies first, or issued
    layer by layer under the attention); and whether the output bits survive the remap."""
    name = "llama8b"
    n_layers = DEFAULT_LAYERS[name]
    wl = Workload(E, torch, W, name, n_layers, 10 * steps + 8, host_for_quarter=True, extra_chunks=512)
    cfg, pool, ids, Tc, B = wl.cfg, wl.pool, wl.ids, wl.cfg.tokens_per_chunk, wl.cfg.batch
    sel = list(range(0, B, 4))

    def slots(b, extra=0):
        return int(-(-(int(wl.lens[b]) + extra) // Tc))

    # Which chunks a fetch goes into is the caller's choice. Left to the pool it is the lowest free ids,
    # which here are the ones an offload has just let go of and is still reading: the fetch then waits
    # for that offload and the two directions take turns. With `oldest_first` the step keeps its own
    # list of free KV chunks in the order they became free and fetches into the ones free the longest.
    free_fifo = []
    oldest_first = [False]

    def refill_fifo():
        owner, state, _, _ = E.ellm_pool_get_owner_state(pool)
        free_now = set(np.flatnonzero((owner == E.ELLM_OWNER_KV) & (state == E.ELLM_CHUNK_FREE)).tolist())
        kept = [c for c in free_fifo if c in free_now]
        known = set(kept)
        free_fifo[:] = sorted(free_now - known) + kept      # chunks not seen before count as free the longest

    def offload_layer(l, extra=0):
        for b in sel:
            n = slots(b, extra)
            if oldest_first[0]:
                tab = E.ellm_tensor_get_table(pool, int(ids[l][b]))[0][:n]
                free_fifo.extend(int(c) for c in tab if c >= 0)
            E.ellm_chunk_deflate_to_host(pool, int(ids[l][b]), 0, n)

    def fetch_layer(l):
        for b in sel:
            n = slots(b)
            if oldest_first[0] and len(free_fifo) >= n + 128:
                want = np.array(free_fifo[:n], np.int32)
                if E.ellm_chunk_inflate_from_host(pool, int(ids[l][b]), 0, n, want, check=False) == 0:
                    del free_fifo[:n]
                    continue
                refill_fifo()                                   # something else took one of them: start over
            E.ellm_chunk_inflate_from_host(pool, int(ids[l][b]), 0, n)

    def sync():
        E.ellm_pool_sync(pool)
        torch.cuda.synchronize()

    def timed(fn, n=steps):
        sync()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        sync()
        return (time.perf_counter() - t0) * 1e3 / n

    def hand_over():
        # a3 / a9: 30 % of what the activation side still owns goes idle and changes owner
        owner, state, _, _ = E.ellm_pool_get_owner_state(pool)
        act = np.flatnonzero((owner == E.ELLM_OWNER_ACT) & (state == E.ELLM_CHUNK_FREE)).astype(np.int32)
        give = act[: int(0.3 * len(act))]
        t0 = time.perf_counter()
        if len(give):
            E.ellm_pool_transfer(pool, give, E.ELLM_OWNER_KV)
        return (time.perf_counter() - t0) * 1e6, len(give)

    def plain():
        wl.step()

    def blocking():
        # the parked requests come back, the step runs, they go out again: nothing overlaps
        hand_over()
        for l in range(n_layers):
            fetch_layer(l)
        E.ellm_pool_sync(pool)
        wl.step()
        torch.cuda.synchronize()
        for l in range(n_layers):
            offload_layer(l)
        E.ellm_pool_sync(pool)

    def layerwise():
        # the fetch of layer l + 1 is issued before layer l's attention and the offload of layer l right
        # after it, so the copies run on the side streams under the kernels
        hand_over()
        wl.map_ahead()
        fetch_layer(0)
        for l in range(n_layers):
            if l + 1 < n_layers:
                fetch_layer(l + 1)
            wl.layer_call(l)
            offload_layer(l, 1)
        wl.lens[:] += 1
        wl.steps_done += 1

    for _ in range(2):
        wl.step()
    # invariance: decode without appending, round-trip a quarter of the requests through the host, decode again
    q0, B_ = wl.q[0], cfg.batch
    before = torch.empty_like(wl.out[0])
    after = torch.empty_like(wl.out[0])
    E.ellm_decode_attention(pool, ids[0], q0, before)
    tabs = [E.ellm_tensor_get_table(pool, int(ids[0][b]))[0].copy() for b in sel]
    offload_layer(0)
    fetch_layer(0)
    E.ellm_decode_attention(pool, ids[0], q0, after)
    sync()
    moved = sum(int((E.ellm_tensor_get_table(pool, int(ids[0][b]))[0] != tabs[i]).sum()) for i, b in enumerate(sel))
    invariant = bool(torch.equal(before, after))

    t_plain = timed(plain)
    us_hand, n_hand = hand_over()
    nbytes = sum(slots(b) for b in sel) * cfg.chunk_bytes * n_layers
    t_off = timed(lambda: [offload_layer(l) for l in range(n_layers)], 1)      # park the selected requests
    t_fetch = timed(lambda: [fetch_layer(l) for l in range(n_layers)], 1)
    t_off2 = timed(lambda: [offload_layer(l) for l in range(n_layers)], 1)     # parked again: the state between steps
    t_block = timed(blocking)
    # the same with the library's copy kernel instead of the copy engines (the requests are parked at this point)
    E.ellm_debug_set_copy_kernels(pool, 1)
    t_fetch_k = timed(lambda: [fetch_layer(l) for l in range(n_layers)], 1)
    t_off_k = timed(lambda: [offload_layer(l) for l in range(n_layers)], 1)
    t_block_k = timed(blocking)
    E.ellm_debug_set_copy_kernels(pool, 0)
    E.ellm_pool_profile_enable(pool, steps * n_layers)
    E.ellm_pool_profile_stride(pool, 13)
    t_layer = timed(layerwise)
    kern = E.ellm_pool_profile_collect(pool, steps * n_layers)
    E.ellm_pool_profile_enable(pool, 0)
    oldest_first[0] = True
    refill_fifo()
    layerwise()                                                  # one step to get the rotation going
    t_layer_oldest = timed(layerwise)
    oldest_first[0] = False
    for l in range(n_layers):          # leave everything resident
        fetch_layer(l)
    sync()
    n_items, _, n_split_req = wl.n_split_items()
    ab = W.algorithmic_bytes(cfg, wl.lens, n_items)
    partial_bytes = (ab["kv"] + ab["q_out"] // 2 + ab["table"] + ab["partials"] // 2 + ab["append"]
                     + (B_ - n_split_req) * cfg.n_q_heads * cfg.head_dim * 2)
    res = {
        "workload": f"llama8b shapes, {n_layers} layers, every 4th request ({len(sel)} of {B}) offloaded to pinned host and fetched "
                    f"between steps, 30 % of the idle activation chunks handed to the KV side before each step",
        "bytes_each_way_per_step": int(nbytes),
        "attention_kernel_GBps_during_migration": round(partial_bytes / (float(np.mean(kern)) * 1e-3) / 1e9, 1) if len(kern) else None,
        "attention_kernel_us_during_migration": round(float(np.mean(kern)) * 1e3, 2) if len(kern) else None,
        "offload_GBps": round(nbytes / (min(t_off, t_off2) * 1e-3) / 1e9, 2), "fetch_GBps": round(nbytes / (t_fetch * 1e-3) / 1e9, 2),
        "ms_step_no_migration": round(t_plain, 3),
        "ms_step_copies_then_compute": round(t_block, 3), "ms_step_layerwise": round(t_layer, 3),
        "ms_step_layerwise_fetch_into_chunks_free_the_longest": round(t_layer_oldest, 3),
        "with_copy_kernel_instead_of_copy_engines": {"offload_GBps": round(nbytes / t_off_k / 1e6, 2),
                                                     "fetch_GBps": round(nbytes / t_fetch_k / 1e6, 2),
                                                     "ms_step_copies_then_compute": round(t_block_k, 3)},
        "ms_hidden_by_layerwise": round(t_block - t_layer, 3),
        "ownership_transfer_us": round(us_hand, 1), "chunks_handed_over": n_hand,
        "output_bits_unchanged_by_remap": invariant, "slots_remapped_in_check": moved,
    }
    wl.close()
    del wl
    torch.cuda.empty_cache()
    return res


def driver_mapped_compare(E, torch, W, args, K=30, Wm=5):
    """The headline model in a driver-mapped pool (the paper's mechanism: chunks mapped into each tensor's
    address range by the driver, kernels read contiguous addresses): step and kernel time with the kernels
    reading the tensors' ranges and, on the same pool, reading through the software table; what the driver's
    calls cost at set-up and per step."""
    name = "llama8b"
    wl = Workload(E, torch, W, name, DEFAULT_LAYERS[name], 3 * (K + Wm) + 2, pool_kind="driver-mapped")
    E.ellm_pool_sync(wl.pool)
    steps = K + Wm

    def leg():
        s0, w0 = E.ellm_pool_get_mapping_stats(wl.pool), E.ellm_pool_get_mapping_wait(wl.pool)
        r, _, _ = measure(wl, K, Wm, args.event_stride)
        s1, w1 = E.ellm_pool_get_mapping_stats(wl.pool), E.ellm_pool_get_mapping_wait(wl.pool)
        d = {k: r[k] for k in ("value", "ms_per_step", "ms_per_step_median", "us_per_layer")}
        d["maps_per_step"] = round((s1["maps"] - s0["maps"]) / steps, 2)
        d["driver_us_per_step"] = round((s1["us_map"] - s0["us_map"]) / steps, 1)
        d["caller_waited_us_per_step"] = round((w1 - w0) / steps, 1)
        if r["roofline"]:
            d["attention_kernel_us"] = r["roofline"]["avg_launch_us"]
            d["attention_kernel_frac_of_peak"] = r["roofline"]["frac"]
        return d

    setup = E.ellm_pool_get_mapping_stats(wl.pool)
    # every call waits for its own driver calls, slots are mapped in the step that writes them
    wl.map_lookahead = 0
    E.ellm_debug_set_async_mapping(wl.pool, 0)
    inline = leg()
    E.ellm_debug_set_async_mapping(wl.pool, 1)
    # the pool as it is meant to be used: slots mapped a few steps early, driver calls on the pool's own
    # thread (the first warm-up step maps what the eight steps after it need)
    wl.map_lookahead = 8
    direct = leg()
    # and with the kernels reading through the software table, on the same chunks
    E.ellm_debug_set_table_kernels(wl.pool, 1)
    table = leg()
    E.ellm_debug_set_table_kernels(wl.pool, 0)
    res = {
        "workload": f"llama8b shapes, {wl.n_layers} layers, {wl.n_chunks} chunks created and mapped by the driver",
        "setup": {"slots_mapped": setup["maps"], "us_per_map_and_set_access": round(setup["us_map"] / max(setup["maps"], 1), 2),
                  "host_s_create_tensors_and_map": round(wl.setup_map_s, 3)},
        "kernels_read_tensor_ranges": direct,
        "same_with_driver_calls_made_by_the_caller": inline,
        "kernels_read_through_table": table,
    }
    # unmap: what taking chunks out of a tensor's range costs (destroy one request's tensors in every layer)
    b = int(np.argsort(wl.lens)[wl.cfg.batch // 2])
    torch.cuda.synchronize()
    s2 = E.ellm_pool_get_mapping_stats(wl.pool)
    for l in range(wl.n_layers):
        E.ellm_tensor_destroy(wl.pool, int(wl.ids[l][b]))
    s3 = E.ellm_pool_get_mapping_stats(wl.pool)
    res["us_per_unmap"] = round((s3["us_unmap"] - s2["us_unmap"]) / max(s3["unmaps"] - s2["unmaps"], 1), 2)
    wl.close()
    del wl
    torch.cuda.empty_cache()
    return res


# ------------------------------------------------------------------------------------------------------
def under_profiler():
    """rocprofv3 (and its predecessors) announce themselves in the environment of the program they run."""
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ):
        return True
    return "rocprof" in os.environ.get("LD_PRELOAD", "").lower()


def run_in_processes(args):
    """The default run: the headline workload and each of the other workloads in a process of its own, one
    after the other; their figures are merged into the one line this process prints. A workload then sees
    the GPU as a fresh process finds it, and this process can leave the GPU idle between two of them (see
    IDLE_BEFORE below). This process starts the others before anything in it has touched the GPU, and
    never does."""
    import subprocess

    def child(extra, timeout):
        cmd = [sys.executable, os.path.abspath(__file__), "--gpus", "1", *extra]
        try:
            r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=timeout, cwd=ROOT)
        except subprocess.TimeoutExpired:
            return None, f"no result within {timeout} s"
        sys.stderr.write(r.stderr[-4000:])
        lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
        if r.returncode != 0 or not lines:
            return None, f"exit status {r.returncode}: {r.stderr.strip()[-300:]}"
        return json.loads(lines[-1]), None

    def memory_temperature():
        """HBM temperature in degrees C as the driver's tool reports it, or None."""
        try:
            out = subprocess.run(["rocm-smi", "--showtemp", "--json"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL,
                                 text=True, timeout=15).stdout
            doc = json.loads([l for l in out.splitlines() if l.startswith("{")][-1])
            vals = [float(v) for card in doc.values() for k, v in card.items() if "memory" in k.lower()]
            return max(vals) if vals else None
        except Exception:
            return None

    # A workload that follows another does not find the GPU as the first one does: for some seconds after a
    # process that held tens of GB of device memory has let go of them, kernels of the next process move
    # 4-8 % fewer bytes per second (the 13B-shaped layer: 3.31 ms on a GPU that has been idle, 3.46-3.58 ms
    # right after another large workload has ended, 3.31 ms again after 20-25 s), and copies over PCIe are
    # slower as well. It is not the heat: the same layer takes 3.33 ms after three seconds of reading at
    # full rate, HBM sensor at 57 degrees, and the 8B-shaped step takes the same time warm or cool (the line
    # carries that measurement too). Something is still at work on the memory that was given back. So that
    # every workload is measured as on an idle GPU, the GPU is left idle for IDLE_BEFORE seconds first, and
    # until the HBM sensor is back to within 3 degrees of its first reading; the idle times and the sensor's
    # readings go into the line.
    IDLE_BEFORE = {"headline": 20.0, "long70b": 20.0, "mha13b": 20.0}
    t_start = memory_temperature()
    temps, idled = {}, {}

    def cooled(at_least, patience=40.0):
        t0 = time.perf_counter()
        if at_least > 0:
            time.sleep(at_least)
        t = memory_temperature()
        while t is not None and t_start is not None and t > t_start + 3.0 and time.perf_counter() - t0 < patience:
            time.sleep(2.0)
            t = memory_temperature()
        return t, round(time.perf_counter() - t0, 1)

    passed = ["--steps", str(args.steps), "--warmup", str(args.warmup)]
    for flag, on in (("--no-cpu-baseline", args.no_cpu_baseline), ("--no-kernel-events", args.no_kernel_events),
                     ("--no-ceilings", args.no_ceilings), ("--separate-calls", args.separate_calls),
                     ("--turnover", args.turnover), ("--vmm-latency", args.vmm_latency)):
        if on:
            passed.append(flag)
    if args.event_stride:
        passed += ["--event-stride", str(args.event_stride)]
    if args.placement != "shuffled":
        passed += ["--placement", args.placement]
    if args.prefill_append:
        passed += ["--prefill-append", str(args.prefill_append)]
    # whatever ran on the GPU before this program (tests, another benchmark) is given time to wear off too
    t_head, idled["headline"] = cooled(IDLE_BEFORE["headline"])
    res, err = child(["--config", args.config, "--no-extras", *passed], 900)
    if res is None:
        print("bench.py: the headline measurement failed: " + err, file=sys.stderr)
        return 1
    temps["headline"] = [t_head, memory_temperature()]
    workloads = {}
    # the headline workload once more, this time after three seconds of reading at full rate (the HBM
    # sensor then shows 55-60 degrees instead of 35): what a service that never lets the GPU rest gets
    got, err = child(["--config", args.config, "--no-extras", "--no-cpu-baseline", "--no-ceilings", "--preheat", "3",
                      "--steps", str(args.steps), "--warmup", str(args.warmup)], 600)
    if got is not None:
        keep = ("value", "pct_of_peak", "ms_per_step", "ms_per_step_median", "ms_per_step_p10", "ms_per_step_p90")
        workloads["headline_after_3s_at_full_rate"] = {k: got[k] for k in keep}
        if got.get("roofline"):
            workloads["headline_after_3s_at_full_rate"]["attention_kernel_us"] = got["roofline"]["avg_launch_us"]
            workloads["headline_after_3s_at_full_rate"]["attention_kernel_frac_of_peak"] = got["roofline"]["frac"]
    else:
        workloads["headline_after_3s_at_full_rate"] = {"error": err}
    temps["headline_after_3s_at_full_rate"] = [None, memory_temperature()]
    for name in LEGS:
        leg_flags = ["--leg", name] + (["--no-ceilings"] if args.no_ceilings else [])
        before, idled[name] = cooled(IDLE_BEFORE.get(name, 0.0))
        got, err = child(leg_flags, 600)
        temps[name] = [before, memory_temperature()]
        workloads[name] = got if got is not None else {"error": err}
    res["workloads"] = workloads
    res["hbm_temperature_C_before_and_after"] = temps
    res["seconds_idle_before"] = idled
    res["config"]["workload"] += ("; also, under `workloads`: long70b and mha13b layers measured the same way, the elastic step "
                                  "(ownership transfer + offload / fetch of every 4th request) and the same model in a "
                                  "driver-mapped pool; every workload in a process of its own")
    print(json.dumps(res))
    return 0


# ------------------------------------------------------------------------------------------------------
def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(the path needs no collective and nothing in it spans GPUs)", file=sys.stderr)
        sys.exit(2)
    extras = args.extras if args.extras is not None else (args.config == "llama8b" and args.pool == "plain"
                                                          and args.pool_memory == "malloc" and not args.split
                                                          and not args.waves_percent and not args.layers
                                                          and not args.leg)
    if extras and under_profiler():
        # a profiled program must not start other programs (the profiler has initialised the GPU in this
        # process already): only the headline workload then, in this process
        print("bench.py: running under a profiler: only the headline workload is measured, in this process "
              "(same as --no-extras)", file=sys.stderr)
        extras = False
    if extras:
        # every workload in a process of its own, one after the other, started by this one, which never
        # touches the GPU itself (see run_in_processes)
        sys.exit(run_in_processes(args))
    # the oracle's library is loaded (and, if it is missing, compiled: a child process) before anything
    # in this process touches the GPU
    from oracle import model as _oracle_model
    _oracle_model.load()
    import torch
    import paper_2506_15155_amd as E
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.leg:
        fn = {"elastic": lambda: elastic_step(E, torch, W, args),
              "driver_mapped": lambda: driver_mapped_compare(E, torch, W, args),
              "long70b": lambda: sub_workload(E, torch, W, "long70b", 20, 5, args, 3),
              "mha13b": lambda: sub_workload(E, torch, W, "mha13b", 20, 5, args, 4)}[args.leg]
        print(json.dumps(fn()))
        return
    K, Wm = args.steps, args.warmup
    if args.config in ("mha13b", "long70b"):
        K, Wm = min(K, 20), min(Wm, 5)
    n_layers = args.layers or DEFAULT_LAYERS[args.config]
    oracle_leg = not args.no_cpu_baseline
    extra_chunks = 0
    cfg = W.CONFIGS[args.config]
    if args.prefill_append:
        extra_chunks = n_layers * cfg.batch * -(-args.prefill_append // cfg.tokens_per_chunk)
    wl = Workload(E, torch, W, args.config, n_layers, K + Wm, pool_kind=args.pool, pool_memory=args.pool_memory,
                  placement=args.placement, keep_hist_for=(0,) if oracle_leg else (), split=args.split,
                  waves_percent=args.waves_percent, extra_chunks=extra_chunks,
                  extra_tensors=n_layers * cfg.batch if args.prefill_append else 0)
    wl.fused = not args.separate_calls
    head, ab, partial_bytes = measure(wl, K, Wm, args.event_stride, not args.no_kernel_events, args.preheat)
    roofline = head.pop("roofline")
    if roofline is not None and not args.no_ceilings:
        roofline.update(read_ceilings(wl, partial_bytes, ab["kv"]))
        roofline["frac_of_measured_read_ceiling"] = round(roofline["achieved"] / roofline["contiguous_read_GBps"], 4)
    if roofline is not None and args.pool == "plain" and not args.split and not args.waves_percent:
        roofline["traffic"], src = committed_traffic(args.config)
        if src:
            roofline["traffic_source"] = src

    parity = cpu = None
    if oracle_leg:
        threads = host_threads()
        B = cfg.batch
        if args.config in ("llama8b", "tiny"):
            sample = list(range(B))
        else:
            order = np.argsort(wl.lens, kind="stable")
            sample = sorted(int(order[r]) for r in np.unique(np.rint(np.linspace(0, B - 1, 4)).astype(int)))
        parity, orc, oids = parity_check(wl, 0, sample, threads)
        if len(sample) == B:
            cpu = cpu_baseline(wl, orc, oids, threads)
        orc.close()

    turn = time_turnover(E, torch, wl) if args.turnover else None
    pre = time_prefill_append(E, torch, wl, args.prefill_append) if args.prefill_append else None

    Hq, Hkv, D, B = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.batch
    desc = (f"{args.config}: {Hq}q/{Hkv}kv heads, head_dim {D}, batch {B}, {n_layers} layers, "
            f"lengths {cfg.length_dist} {cfg.len_lo}..{cfg.len_hi} (mean {head['mean_context']:.0f}), "
            f"{cfg.chunk_bytes >> 10} KiB chunks "
            + ("shuffled" if args.placement == "shuffled" else "in consecutive runs per tensor")
            + f" in one pool of {wl.n_chunks}"
            + (" (each chunk a physical allocation of its own, driver-mapped)" if args.pool_memory == "vmm" else "")
            + ({"plain": "", "driver-mapped": " (driver-mapped pool, kernels read the tensors' address ranges)",
                "driver-mapped-table-kernels": " (driver-mapped pool read through the table)"}[args.pool])
            + ", step = per layer map-ahead + append 1 token/request + decode"
            + (" (one fused call)" if wl.fused else " (two calls)"))
    n_chunks_head = wl.n_chunks
    wl.close()
    del wl
    torch.cuda.empty_cache()

    res = {
        "metric": METRIC, "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "pct_of_peak": head["pct_of_peak"], "tokens_per_s": head["tokens_per_s"],
        "tokens_per_s_per_layer": head["tokens_per_s_per_layer"],
        "ms_per_step_median": head["ms_per_step_median"], "ms_per_step_p10": head["ms_per_step_p10"],
        "ms_per_step_p90": head["ms_per_step_p90"],
        "value_without_partials": head["value_without_partials"], "value_kv_only": head["value_kv_only"],
        "config": {"workload": desc, "global_batch": B, "layers": n_layers, "split_tokens": head["split_tokens"],
                   "partials_per_kv_head": head["partials_per_kv_head"],
                   "requests_finished_by_the_attention_kernel": head["requests_finished_by_the_attention_kernel"],
                   "algorithmic_bytes_per_step": head["algorithmic_bytes_per_step"], "pool_chunks": n_chunks_head},
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity,
    }
    if pre:
        res["prefill_append"] = pre
    if turn:
        res["turnover"] = turn
    if args.vmm_latency:
        rc, us = E.ellm_debug_vmm_latency(cfg.chunk_bytes, 256, check=False)
        res["vmm_us_per_chunk"] = ({"create": round(us[0], 2), "map_and_set_access": round(us[1], 2), "unmap": round(us[2], 2),
                                    "release": round(us[3], 2), "chunks": 256} if rc == 0
                                   else {"error": E.ellm_last_error()})
    print(json.dumps(res))


def time_turnover(E, torch, wl, rounds=20):
    """Host cost of replacing a finished request by a new one of the same prompt length in every layer:
    (a) release + acquire, where the best-fitting available tensor is taken with its mapping intact and
    no table entry changes; (b) destroy + create + map, where every slot is mapped again and the device
    table has to be patched. Microseconds per request and layer; the tensors end up as they started."""
    cfg, pool, ids, lens, n_layers, max_tokens = wl.cfg, wl.pool, wl.ids, wl.lens, wl.n_layers, wl.max_tokens
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
                ids[l][b] = E.ellm_tensor_acquire(pool, need, max_tokens)
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
    return {"us_release_plus_best_fit_acquire": round(t_reuse / n_ops * 1e6, 2),
            "us_destroy_create_map": round(t_remap / n_ops * 1e6, 2),
            "slots_per_request": [int(-(-int(lens[b]) // Tc)) for b in pick],
            "note": "host time per request and layer through the Python binding; the second path also leaves one "
                    "table entry per slot to be patched on the device by the next call"}


def time_prefill_append(E, torch, wl, n_tok):
    """Multi-token append (the prefill-side write): n_tok tokens per request into fresh tensors of every
    layer; GB/s counts the new K/V rows read and written."""
    cfg, pool, n_layers, max_tokens = wl.cfg, wl.pool, wl.n_layers, wl.max_tokens
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
