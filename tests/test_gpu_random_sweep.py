"""Seeded random sweep: table shape, probe depth, policy, retention, batch size and id mix drawn
at random; every call compared with the oracle bit for bit (out_slots, evicted set, counters,
identities, metadata)."""
import os

import numpy as np
import pytest

from paper_2602_17050_amd import workloads as wl
from gpu_common import Pair, say

pytestmark = pytest.mark.gpu

POLICIES = [True, False, "lru", "expiry"]


def draw_ids(rng, n, universe):
    kind = int(rng.integers(0, 6))
    if kind == 0:
        return wl.zipf_ids(rng, n, 1.05 + 0.3 * float(rng.random()), universe)
    if kind == 1:
        return rng.integers(0, universe, size=n)
    if kind == 2:
        return rng.integers(-4, universe, size=n)                          # some invalid ids
    if kind == 3:
        return wl.rank_to_id(rng.integers(universe, 4 * universe, size=n))  # mostly unseen ids
    if kind == 4:
        return np.full(n, int(rng.integers(0, universe)))                  # one id, many copies
    return np.repeat(rng.integers(0, universe, size=max(n // 7, 1)), 7)[:n]  # runs of equal ids


# MPZCH_SWEEP_BLOCKS widens the sweep for an occasional long run (16 tables per block)
@pytest.mark.parametrize("block", range(int(os.environ.get("MPZCH_SWEEP_BLOCKS", "12"))))
def test_random_tables_every_policy(block):
    rng = np.random.Generator(np.random.Philox(key=0x5EED + block))
    for case in range(16):
        policy = POLICIES[int(rng.integers(0, 4))]
        n_slots = int(rng.choice([1, 2, 3, 15, 16, 17, 63, 64, 65, 200, 1000, 5000]))
        p_hi = 300
        max_probe = int(rng.choice([1, 2, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, p_hi]))
        ttl = int(rng.integers(0, 4))
        universe = max(2, int(n_slots * float(rng.choice([0.5, 1.5, 4.0]))))
        # every other table is kept as one tensor of 16-byte records
        p = Pair(n_slots, max_probe, ttl, policy, hash_seed=int(rng.integers(0, 1 << 62)),
                 layout="records" if case % 2 else "separate")
        step = int(rng.integers(0, 5))
        for k in range(int(rng.integers(3, 7))):
            n = int(rng.choice([0, 1, 63, 64, 65, 500, 4097])) if rng.random() < 0.5 else int(rng.integers(0, 6 * n_slots + 2))
            ids = draw_ids(rng, n, universe) if n else np.empty(0, np.int64)
            ttls = None
            if policy == "expiry" and rng.random() < 0.7:
                if rng.random() < 0.5:
                    # the retention belongs to the id's feature: all copies of an id carry the same value
                    ttls = ((np.asarray(ids, dtype=np.int64) >> 3) % 5).astype(np.int32)
                else:
                    ttls = rng.integers(0, 5, size=len(ids)).astype(np.int32)    # copies of an id disagree
            say("sweep block", block, "case", case, "policy", policy, "N", n_slots, "P", max_probe, "ttl", ttl,
                "step", step, "n", len(ids))
            p.step(ids, step, ttls=ttls)
            assert p.o.check_state()[0] == 0
            step += int(rng.integers(0, 3))
        p.lookup(rng.integers(-2, 2 * universe, size=300))
        p.close()


@pytest.mark.parametrize("block", range(int(os.environ.get("MPZCH_SWEEP_BLOCKS", "12"))))
def test_random_groups_of_tables(block):
    """Keyed jagged batches over 1..8 tables of random shape and policy, through one group."""
    from test_gpu_jagged import JaggedPair

    rng = np.random.Generator(np.random.Philox(key=0xFACE + block))
    for case in range(6):
        T = int(rng.integers(1, 9))
        specs = []
        for f in range(T):
            policy = POLICIES[int(rng.integers(0, 4))]
            n_slots = int(rng.choice([1, 2, 17, 64, 65, 300, 2000]))
            max_probe = int(rng.choice([1, 3, 8, 9, 16, 17, 32, 33, 64, 150]))
            specs.append(wl.TableSpec(n_slots, max_probe, int(rng.integers(0, 4)), policy, int(rng.integers(0, 1 << 40))))
        jp = JaggedPair(specs)
        step = int(rng.integers(0, 4))
        for k in range(int(rng.integers(2, 6))):
            counts = [0 if rng.random() < 0.2 else int(rng.integers(0, 5 * s.num_slots + 3)) for s in specs]
            vals = [draw_ids(rng, c, max(2, 3 * s.num_slots)) if c else np.empty(0, np.int64) for s, c in zip(specs, counts)]
            values = np.concatenate(vals).astype(np.int64)
            offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
            say("group sweep block", block, "case", case, "step", step, "tables",
                [(s.num_slots, s.max_probe, s.evict) for s in specs], "counts", counts)
            jp.step(values, offsets, step)
            jp.check_state()
            jp.lookup(values, offsets)
            step += int(rng.integers(0, 3))
        for o in jp.o:
            assert o.check_state()[0] == 0
        jp.close()
