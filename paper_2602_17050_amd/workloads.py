"""Seeded synthetic ID streams shaped like the paper's workloads.

This module only *draws inputs*: it holds none of the method's arithmetic
(no hashing to slots, no probing, no eviction) and is the one piece of code
that both the HIP path's tests/benchmark and the CPU oracle's tests consume.

The paper's own streams are production ID logs (150 M user IDs behind Table 1;
post / owner IDs in Sec. 4) that cannot be reproduced; what is kept is their
shape: heavy-tailed (Zipf-like) popularity, a steady churn of brand-new item
IDs with decaying popularity of old ones, and table-size : cardinality ratios
like those of Table 1.

Everything is drawn from numpy's counter-based Philox generator keyed by
``DATA_SEED + 1000 * config + step`` so that any batch can be regenerated
independently of the others.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

DATA_SEED = 20260217
HASH_SEED_BASE = 0x5EED0000

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_MASK63 = np.uint64((1 << 63) - 1)

NEW_ID_BASE = 1 << 40        # monotone counter ids of the streaming configs
PREFILL_ID_BASE = 1 << 41    # prefill ids of the streaming configs (disjoint from the above)
PREFILL_RANK_BASE = 1 << 42  # ranks (before scattering) of prefill ids of the Zipf configs


def rng_for(config: int, step: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=DATA_SEED + 1000 * config + step))


def rank_to_id(rank: np.ndarray) -> np.ndarray:
    """Bijection of [0, 2^63): scatters small ranks over the non-negative int64 range."""
    r = np.asarray(rank).astype(np.uint64)
    with np.errstate(over="ignore"):
        return ((r * _GOLDEN) & _MASK63).astype(np.int64)


def zipf_ranks(rng: np.random.Generator, n: int, alpha: float, universe: int) -> np.ndarray:
    """n ranks in [1, universe], P(rank = k) roughly proportional to k^-alpha.

    Inverse CDF of the bounded Pareto density on [1, universe + 1), floored.
    """
    u = rng.random(n)
    one_m = 1.0 - alpha
    top = float(universe + 1) ** one_m
    x = ((top - 1.0) * u + 1.0) ** (1.0 / one_m)
    return np.minimum(np.floor(x), universe).astype(np.int64)


def zipf_ids(rng, n, alpha, universe):
    return rank_to_id(zipf_ranks(rng, n, alpha, universe))


def scattered_prefill_ids(lo: int, hi: int) -> np.ndarray:
    """Distinct ids, disjoint from every Zipf universe used here (ranks start at 2^42)."""
    return rank_to_id(np.arange(lo, hi, dtype=np.int64) + PREFILL_RANK_BASE)


def fresh_uniform_ids(rng: np.random.Generator, n: int) -> np.ndarray:
    """Uniform 63-bit values (practically never resident)."""
    return (rng.integers(0, 1 << 63, size=n, dtype=np.uint64) & _MASK63).astype(np.int64)


# --------------------------------------------------------------------------
# Table / embedding descriptions
# --------------------------------------------------------------------------
@dataclass
class TableSpec:
    num_slots: int
    max_probe: int
    ttl: int               # steps; ignored when evict is False
    evict: object = True   # True = TTL eviction, False = off; tests also pass "lru" / "expiry"
    hash_seed: int = HASH_SEED_BASE
    emb_rows: int = 0      # rows of the embedding the reset targets (row = slot mod emb_rows)
    emb_dim: int = 0
    emb_dtype: str = "float32"


# --------------------------------------------------------------------------
# Config 1: tiny table, 8 Zipf batches, TTL 3
# --------------------------------------------------------------------------
def c1_spec() -> TableSpec:
    return TableSpec(4096, 8, 3, True, HASH_SEED_BASE, 4096, 16, "float32")


def c1_batches():
    """[(step, ids int64[1024])] for steps 1..8, Zipf(1.1) over 16 384 ids."""
    return [(s, zipf_ids(rng_for(1, s), 1024, 1.1, 16384)) for s in range(1, 9)]


# --------------------------------------------------------------------------
# Config 2: 1 M slots, load 0.3 -> ~0.9, TTL 10
# --------------------------------------------------------------------------
C2_FRESH_PER_BATCH = 3277  # 5 % of the batch are never-seen ids so that the table keeps filling


def c2_spec() -> TableSpec:
    return TableSpec(1_000_000, 16, 10, True, HASH_SEED_BASE + 1, 1_000_000, 64, "float32")


def c2_prefill():
    """(step 0, 300 000 distinct ids outside the Zipf universe) -> load 0.30."""
    return 0, scattered_prefill_ids(0, 300_000)


def c2_batch(step: int, n: int = 65536) -> np.ndarray:
    rng = rng_for(2, step)
    ids = zipf_ids(rng, n, 1.05, 2_000_000)
    k = C2_FRESH_PER_BATCH * n // 65536
    pos = rng.choice(n, size=k, replace=False)
    ids[pos] = scattered_prefill_ids(10_000_000 + step * k, 10_000_000 + (step + 1) * k)
    return ids


# --------------------------------------------------------------------------
# Config 3: read-only lookups on a prefilled table
# --------------------------------------------------------------------------
def c3_spec(num_slots: int = 100_000_000) -> TableSpec:
    return TableSpec(num_slots, 32, 0, False, HASH_SEED_BASE + 2)


def c3_prefill_ids(lo: int, hi: int) -> np.ndarray:
    return scattered_prefill_ids(lo, hi)


def c3_batch(step: int, n: int, num_resident_ids: int) -> np.ndarray:
    """95 % Zipf(1.2) over the prefilled ids (popularity order is a seeded
    permutation of insertion order), 5 % uniform 63-bit ids that are not resident."""
    rng = rng_for(3, step)
    n_miss = n // 20
    ranks = zipf_ranks(rng, n - n_miss, 1.2, num_resident_ids) - 1
    # fixed odd-multiplier permutation of [0, num_resident_ids): popularity rank -> insertion index
    idx = (ranks.astype(np.uint64) * np.uint64(2654435761) + np.uint64(12345)) % np.uint64(num_resident_ids)
    ids = np.concatenate([rank_to_id(idx.astype(np.int64) + PREFILL_RANK_BASE),
                          fresh_uniform_ids(rng, n_miss)])
    rng.shuffle(ids)
    return ids


# --------------------------------------------------------------------------
# Streaming-freshness stream (config 4 and the 1 B-slot headline)
# --------------------------------------------------------------------------
@dataclass
class StreamSpec:
    table: TableSpec
    config: int             # seed namespace
    prefill_ids: int        # ids inserted at step 0: PREFILL_ID_BASE + [0, prefill_ids)
    batch: int              # ids per step
    first_step: int         # first streamed step (ttl + 1: the prefill is expired from here on)
    new_fraction: float = 0.10
    mean_age: float = 10.0


def c4_spec(scale: float = 1.0) -> StreamSpec:
    n = int(500_000_000 * scale)
    t = TableSpec(n, 16, 20, True, HASH_SEED_BASE + 3, max(int(100_000_000 * scale), 1), 128, "bfloat16")
    return StreamSpec(t, 4, int(0.9 * n), max(int(2_000_000 * scale), 64), 21)


def headline_spec(scale: float = 1.0) -> StreamSpec:
    n = int(1_000_000_000 * scale)
    t = TableSpec(n, 16, 20, True, HASH_SEED_BASE + 5, max(int(100_000_000 * scale), 1), 128, "bfloat16")
    return StreamSpec(t, 6, int(0.7 * n), max(int(4_000_000 * scale), 64), 21)


def stream_prefill_ids(lo: int, hi: int) -> np.ndarray:
    return np.arange(lo, hi, dtype=np.int64) + PREFILL_ID_BASE


def stream_batch(spec: StreamSpec, step: int) -> np.ndarray:
    """One step of the freshness stream.

    ``new_fraction`` of the batch are brand-new ids from a monotone counter; the
    rest re-visit old ids: draw an age a >= 1 (geometric, mean ``mean_age``
    steps) and pick uniformly among the ids that were new at step - a, or among
    the prefill ids when that lies before the stream began.
    """
    rng = rng_for(spec.config, step)
    n = spec.batch
    m = int(round(n * spec.new_fraction))
    k = step - spec.first_step
    new_ids = NEW_ID_BASE + k * m + np.arange(m, dtype=np.int64)
    n_old = n - m
    age = rng.geometric(1.0 / spec.mean_age, size=n_old).astype(np.int64)
    born = k - age                                   # stream step index the id was new at
    u = rng.random(n_old)
    from_stream = born >= 0
    old = np.empty(n_old, dtype=np.int64)
    old[from_stream] = NEW_ID_BASE + born[from_stream] * m + (u[from_stream] * m).astype(np.int64)
    old[~from_stream] = PREFILL_ID_BASE + (u[~from_stream] * spec.prefill_ids).astype(np.int64)
    ids = np.concatenate([new_ids, old])
    rng.shuffle(ids)
    return ids


# --------------------------------------------------------------------------
# Config 5: 26 tables, keyed jagged batch
# --------------------------------------------------------------------------
@dataclass
class JaggedSpec:
    tables: list = field(default_factory=list)     # TableSpec per feature
    pooling: list = field(default_factory=list)    # pooling factor per feature
    samples: int = 65536


def c5_spec(total_slots_cap: int = 1_000_000_000, samples: int = 65536, num_tables: int = 26,
            emb_dim: int = 16) -> JaggedSpec:
    rng = rng_for(5, 0)
    raw = 10.0 ** rng.uniform(3.0, 9.0, size=num_tables)
    scale = min(1.0, total_slots_cap / float(raw.sum()))
    slots = np.maximum((raw * scale).astype(np.int64), 1000)
    pooling = rng.integers(1, 51, size=num_tables)
    tables = [TableSpec(int(slots[f]), 16, 5, True, HASH_SEED_BASE + 100 + f, int(slots[f]), emb_dim, "bfloat16")
              for f in range(num_tables)]
    return JaggedSpec(tables, [int(p) for p in pooling], samples)


def c5_batch(spec: JaggedSpec, step: int):
    """Feature-major keyed jagged batch.

    Returns (values int64[total], lengths int32[num_tables * samples],
    feature_offsets int64[num_tables + 1]).  Per sample and feature the length is
    uniform on [0, 2 * pooling]; ids are Zipf(1.05) over a universe twice the
    table's slot count.
    """
    rng = rng_for(5, step + 1)
    vals, lens, offs = [], [], [0]
    for f, (t, pf) in enumerate(zip(spec.tables, spec.pooling)):
        ln = rng.integers(0, 2 * pf + 1, size=spec.samples).astype(np.int32)
        cnt = int(ln.sum())
        vals.append(zipf_ids(rng, cnt, 1.05, 2 * t.num_slots))
        lens.append(ln)
        offs.append(offs[-1] + cnt)
    return (np.concatenate(vals) if vals else np.empty(0, np.int64),
            np.concatenate(lens) if lens else np.empty(0, np.int32),
            np.asarray(offs, dtype=np.int64))


# --------------------------------------------------------------------------
# Table-1 style input: n distinct ids (collision-rate experiments)
# --------------------------------------------------------------------------
def distinct_ids(n: int, salt: int = 0) -> np.ndarray:
    return rank_to_id(np.arange(1, n + 1, dtype=np.int64) + (salt << 44))


def distinct_ids_device(lo: int, hi: int, device, salt: int = 0):
    """distinct_ids(n)[lo:hi] drawn on the device (same integers: the multiplication wraps mod 2^64)."""
    import torch
    r = torch.arange(lo + 1, hi + 1, dtype=torch.int64, device=device) + (salt << 44)
    return (r * torch.tensor(-7046029254386353131, dtype=torch.int64, device=device)) & ((1 << 63) - 1)


def embedding_pattern(rows: int, dim: int, dtype=np.float32) -> np.ndarray:
    """Non-zero closed-form fill so that a reset row is observable: integers 1..251."""
    r = np.arange(rows, dtype=np.int64)[:, None]
    c = np.arange(dim, dtype=np.int64)[None, :]
    return ((r * 131 + c * 7) % 251 + 1).astype(dtype)
