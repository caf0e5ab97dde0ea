"""Seeded synthetic inputs for the chunk-backed decode-attention path.

This module only draws random numbers and packages them: shapes, context lengths, chunk
placements, ownership masks and bf16 bit patterns. It holds none of the method's arithmetic (no
attention, no table translation, no pool logic) and imports neither the HIP binding nor the
oracle, so both can be fed from it.

The workloads stand in for the ones the eLLM paper (arXiv 2506.15155) measures on: the long-tailed
prompt lengths of its conversational dataset (Introduction, "Prefill phase"), its fixed-length
2K-2K runs and its 128k-4k long-context run (Sec. 4.4). None of those datasets is used here; only
the length mix and the layer shapes are imitated.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20250615


@dataclass
class Config:
    """One benchmark / test configuration (shapes only)."""
    name: str
    index: int                 # 1-based position in the configuration list
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    chunk_bytes: int
    n_chunks: int              # pool size in chunks
    max_tokens: int            # virtual range of every request
    length_dist: str           # "uniform" | "lognormal"
    len_lo: int
    len_hi: int
    lognormal_median: int = 1024
    lognormal_sigma: float = 1.0
    act_fraction: float = 0.0  # share of pool chunks owned (and held busy) by activations
    host_slots: int = 0

    @property
    def bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2

    @property
    def tokens_per_chunk(self) -> int:
        return self.chunk_bytes // self.bytes_per_token

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def max_slots(self) -> int:
        return -(-self.max_tokens // self.tokens_per_chunk)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


MiB = 1 << 20

CONFIGS = {
    # 1 layer, batch 4, 8 q = 8 kv heads, D 64, 16-token chunks scattered in a 64-chunk pool
    "tiny": Config("tiny", 1, 4, 8, 8, 64, 16 * (2 * 8 * 64 * 2), 64, 256, "uniform", 16, 256),
    # Llama-3-8B-shaped layer: 32 q / 8 kv heads, D 128, batch 64, lognormal lengths, 2 MiB chunks
    "llama8b": Config("llama8b", 2, 64, 32, 8, 128, 2 * MiB, 1024, 8192 + 512, "lognormal", 64, 8192,
                      host_slots=128),
    # 13B-shaped MHA layer: 40 q = 40 kv heads, batch 128, lengths 2k..16k, half the pool is activations
    "mha13b": Config("mha13b", 3, 128, 40, 40, 128, 2 * MiB, 23552, 16384 + 102, "uniform", 2048, 16384,
                     act_fraction=0.5),
    # elastic step: config-2 shapes with an activation region to borrow from and a host buffer
    "elastic": Config("elastic", 4, 64, 32, 8, 128, 2 * MiB, 1024, 8192 + 512, "lognormal", 64, 8192,
                      act_fraction=0.3, host_slots=256),
    # 70B-shaped long-context layer: 64 q / 8 kv heads, batch 16, lengths 32k..128k
    "long70b": Config("long70b", 5, 16, 64, 8, 128, 2 * MiB, 4096, 131072 + 512, "uniform", 32768, 131072),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of cfg with some fields replaced (used for reduced-size parity cases)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return Config(**d)


def draw_lengths(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    """Context lengths AFTER the step's append, one per request."""
    if cfg.length_dist == "uniform":
        lens = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.batch)
    elif cfg.length_dist == "lognormal":
        z = rng.standard_normal(cfg.batch)
        lens = np.rint(np.exp(math.log(cfg.lognormal_median) + cfg.lognormal_sigma * z))
        lens = np.clip(lens, cfg.len_lo, cfg.len_hi)
    else:
        raise ValueError(cfg.length_dist)
    lens = lens.astype(np.int64)
    if cfg.name == "tiny" and cfg.batch >= 2:
        # force one request whose appended token opens a new chunk and one that ends exactly on a
        # chunk boundary, so both edges are always exercised
        tc = cfg.tokens_per_chunk
        lens[0] = min(cfg.len_hi, (int(lens[0]) // tc) * tc + 1)
        lens[1] = max(tc, (int(lens[1]) // tc) * tc)
    return lens


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    """N(0,1) samples rounded to bf16, as uint16 bit patterns."""
    return bf16_bits_from_f32(rng.standard_normal(shape, dtype=np.float32))


BF16_NAN = np.uint16(0x7FC0)


@dataclass
class Placement:
    """Where every request's slots live and who owns the rest of the pool."""
    owner: np.ndarray                 # uint8[n_chunks]: 0 = KV, 1 = activation
    act_busy: np.ndarray              # int32 ids of activation chunks held busy
    chunk_ids: list                   # per request: int32[n_slots_needed], shuffled physical ids
    spare_kv: np.ndarray              # KV-owned chunk ids left unassigned (shuffled)


def draw_placement(cfg: Config, lens: np.ndarray, rng: np.random.Generator,
                   extra_slots: int = 0) -> Placement:
    """Scatter every request's chunks over the pool: a seeded permutation of the KV-owned chunk
    ids, dealt out request by request. With act_fraction > 0 a Bernoulli mask first gives that
    share of the pool to activations (interleaved with the KV chunks)."""
    n = cfg.n_chunks
    owner = np.zeros(n, dtype=np.uint8)
    if cfg.act_fraction > 0:
        owner[rng.random(n) < cfg.act_fraction] = 1
    kv_ids = np.flatnonzero(owner == 0).astype(np.int32)
    rng.shuffle(kv_ids)
    tc = cfg.tokens_per_chunk
    need = [int(-(-int(l) // tc)) + extra_slots for l in lens]
    if sum(need) > len(kv_ids):
        raise ValueError(f"pool too small: need {sum(need)} chunks, {len(kv_ids)} KV-owned")
    out, pos = [], 0
    for k in need:
        out.append(kv_ids[pos:pos + k].copy())
        pos += k
    return Placement(owner, np.flatnonzero(owner == 1).astype(np.int32), out, kv_ids[pos:].copy())


@dataclass
class Step:
    """Everything one decode step consumes, on the host, as bf16 bit patterns."""
    cfg: Config
    lens: np.ndarray                  # int64[batch], lengths after the append
    placement: Placement
    k_hist: list = field(default_factory=list)   # per request uint16[len-1][Hkv][D]
    v_hist: list = field(default_factory=list)
    k_new: np.ndarray = None          # uint16[batch][Hkv][D]
    v_new: np.ndarray = None
    q: np.ndarray = None              # uint16[batch][Hq][D]


def draw_step(cfg: Config, seed: int | None = None, with_values: bool = True,
              extra_slots: int = 0) -> Step:
    """Draw lengths, placement and (optionally) all K/V/Q values for one decode step."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    lens = draw_lengths(cfg, rng)
    pl = draw_placement(cfg, lens, rng, extra_slots)
    st = Step(cfg, lens, pl)
    if with_values:
        for l in lens:
            st.k_hist.append(normal_bf16(rng, (int(l) - 1, cfg.n_kv_heads, cfg.head_dim)))
            st.v_hist.append(normal_bf16(rng, (int(l) - 1, cfg.n_kv_heads, cfg.head_dim)))
        st.k_new = normal_bf16(rng, (cfg.batch, cfg.n_kv_heads, cfg.head_dim))
        st.v_new = normal_bf16(rng, (cfg.batch, cfg.n_kv_heads, cfg.head_dim))
        st.q = normal_bf16(rng, (cfg.batch, cfg.n_q_heads, cfg.head_dim))
    return st


def algorithmic_bytes(cfg: Config, lens: np.ndarray, n_items: int = 0) -> dict:
    """Bytes one append + decode pass over one layer has to move, by the formula of the
    measurement plan: K and V read once per kv head, q read and out written, table entries read,
    the new token read and written, split-K partials written then read."""
    E = 2
    Hq, Hkv, D = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    tc = cfg.tokens_per_chunk
    kv = int(sum(2 * int(l) * Hkv * D * E for l in lens))
    qo = int(len(lens) * 2 * Hq * D * E)
    table = int(sum(4 * (-(-int(l) // tc)) for l in lens))
    app = int(len(lens) * 2 * Hkv * D * E * 2)
    part = int(2 * 4 * n_items * Hq * (D + 2))
    return {"kv": kv, "q_out": qo, "table": table, "append": app, "partials": part,
            "decode_total": kv + qo + table + part, "total": kv + qo + table + app + part}
