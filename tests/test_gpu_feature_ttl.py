"""GPU parity of the per-feature TTL mode (metadata = expiry step, retention given per position)."""
import numpy as np
import pytest

from paper_2602_17050_amd import workloads as wl
from gpu_common import Pair, say

pytestmark = pytest.mark.gpu

CASES = [(1, 1, 5, 9, 6), (17, 8, 60, 100, 12), (100, 16, 500, 1000, 12), (300, 40, 2000, 3000, 8),
         (1000, 100, 5000, 5000, 6), (4099, 4, 30000, 20000, 10)]


def _ttl_of(ids):
    """the feature of an id (its retention class) is a function of the id: all copies agree"""
    return (np.abs(ids) % 4).astype(np.int32) * 2


def _ttl_per_position(rng, ids):
    """one table serving several features: the same id arrives with different retention in one batch"""
    return rng.integers(0, 7, size=len(ids)).astype(np.int32)


@pytest.mark.parametrize("case", CASES, ids=[f"N{c[0]}_P{c[1]}" for c in CASES])
def test_feature_ttl_contended_small_tables(case):
    n_slots, max_probe, universe, batch, steps = case
    rng = np.random.Generator(np.random.Philox(key=(hash(case) ^ 0x77) & 0xFFFFFFFF))
    p = Pair(n_slots, max_probe, 1, "expiry", hash_seed=0xFEE0 + n_slots)
    step, ev = 0, 0
    for k in range(steps):
        step += int(rng.integers(0, 3))
        if k % 3 == 0:
            ids = wl.zipf_ids(rng, batch, 1.1, universe)
        elif k % 3 == 1:
            ids = rng.integers(-2, universe, size=batch // 2 + 1)
        else:
            ids = wl.rank_to_id(rng.integers(universe, 3 * universe, size=batch))
        say("feature-ttl case", case, "step", step)
        # one call with the table's own ttl; every other call lets copies of an id disagree
        ttls = None if k == 4 else (_ttl_per_position(rng, ids) if k % 2 else _ttl_of(ids))
        r = p.step(ids, step, ttls=ttls)
        ev += r.stats["evictions"]
        assert p.o.check_state()[0] == 0
    assert ev > 0 or n_slots == 1
    p.close()


def test_feature_ttl_one_million_slots():
    spec = wl.c2_spec()
    p = Pair(spec.num_slots, spec.max_probe, 3, "expiry", spec.hash_seed, wl.embedding_pattern(spec.emb_rows, 8))
    step0, pre = wl.c2_prefill()
    p.step(pre, step0, check_state=False, ttls=_ttl_of(pre))
    tot = 0
    rng = np.random.Generator(np.random.Philox(key=31337))
    for step in range(1, 31):
        ids = wl.c2_batch(step)
        ttls = _ttl_per_position(rng, ids) if step % 2 else _ttl_of(ids)
        tot += p.step(ids, step, check_state=(step % 10 == 0), ttls=ttls).stats["evictions"]
    say("feature-ttl evictions", tot)
    assert tot > 1000
    p.check_state()
    p.close()
