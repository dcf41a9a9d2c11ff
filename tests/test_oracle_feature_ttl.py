"""CPU-only pins of the per-feature TTL mode (Sec. 3.4: "A TTL value is computed based on the current
training timestamp and a user-defined duration ... updated in the metadata tensor whenever an ID is
processed.  Any slot with a metadata value lower than the current timestamp is deemed expired", and
"per-feature TTL configurations for embedding tables that manage multiple distinct features")."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from test_oracle_pins import py_home, ids_with_home


class ExpiryAlg1:
    """Algorithm 1 for one id at a time with meta = now + duration of the id's feature and the
    expiry test of Sec. 3.4 (stored value lower than the current time stamp)."""

    def __init__(self, n_slots, max_probe, seed):
        self.I, self.M = [-1] * n_slots, [-1] * n_slots
        self.N, self.P, self.seed = n_slots, min(max_probe, n_slots), seed

    def lookup_one(self, id_, step, ttl):
        meta = step + ttl
        h = py_home(id_, self.seed, self.N)
        exists = any(self.I[(h + i) % self.N] == id_ for i in range(self.P))
        for i in range(self.P):
            s = (h + i) % self.N
            if self.I[s] == id_ or (self.I[s] == -1 and not exists):
                self.I[s], self.M[s] = id_, meta
                return s, False
            if not exists and self.I[s] != -1 and self.M[s] < step:
                self.I[s], self.M[s] = id_, meta
                return s, True
        self.M[h] = max(self.M[h], meta)        # Case 3 refreshes, it never shortens the resident's retention
        return h, False


@given(st.data())
@settings(max_examples=150, deadline=None)
def test_single_id_batches_equal_algorithm_1_with_expiry_times(data):
    n_slots = data.draw(st.integers(1, 24))
    max_probe = data.draw(st.integers(1, 30))
    seed = data.draw(st.integers(0, 1 << 20))
    universe = data.draw(st.integers(1, 40))
    calls = data.draw(st.lists(st.tuples(st.integers(0, universe), st.integers(0, 2)), min_size=1, max_size=80))
    ref = ExpiryAlg1(n_slots, max_probe, seed)
    t = oracle.Table(n_slots, max_probe, oracle.EVICT_TTL_EXPIRY, 1, seed)
    step = 0
    for id_, dstep in calls:
        step += dstep
        ttl = id_ % 4                                   # the id's feature decides its retention
        slot, evicted = ref.lookup_one(id_, step, ttl)
        r = t.remap([id_], step, [ttl])
        assert r.slots[0] == slot and (len(r.evicted) == 1) == evicted
        assert t.identities.tolist() == ref.I and t.metadata.tolist() == ref.M


@given(st.data())
@settings(max_examples=80, deadline=None)
def test_one_ttl_for_all_equals_the_last_seen_form(data):
    """With one duration T for every id, storing now + T and testing value < now is the same rule as
    storing now and testing now - value > T: same slots, same evictions, metadata shifted by T."""
    n_slots = data.draw(st.integers(1, 40))
    max_probe = data.draw(st.integers(1, 8))
    ttl = data.draw(st.integers(0, 3))
    seed = data.draw(st.integers(0, 99))
    steps = data.draw(st.lists(st.tuples(st.integers(0, 2), st.lists(st.integers(-2, 60), max_size=40)), min_size=1, max_size=8))
    a = oracle.Table(n_slots, max_probe, oracle.EVICT_TTL, ttl, seed)
    b = oracle.Table(n_slots, max_probe, oracle.EVICT_TTL_EXPIRY, ttl, seed)
    step = 0
    for d, batch in steps:
        step += d
        ra = a.remap(batch, step)
        rb = b.remap(batch, step, [ttl] * len(batch)) if len(batch) % 2 else b.remap(batch, step)
        assert np.array_equal(ra.slots, rb.slots) and np.array_equal(ra.evicted, rb.evicted) and ra.stats == rb.stats
        assert np.array_equal(a.identities, b.identities)
        touched = a.metadata >= 0
        assert np.array_equal(a.metadata[touched] + ttl, b.metadata[touched])
        assert (b.metadata[~touched] == -1).all()


def test_two_features_with_different_retention_share_a_table():
    seed, n = 17, 16
    short, long_, new1, new2 = ids_with_home(9, seed, n, 4)
    t = oracle.Table(n, 2, oracle.EVICT_TTL_EXPIRY, 0, seed)
    r = t.remap([short, long_], 2, [1, 10])                 # window 9, 10 is full now
    assert r.slots.tolist() == [9, 10] and t.metadata[9] == 3 and t.metadata[10] == 12
    r = t.remap([new1], 3, [1])                             # nothing expired yet: 3 < 3 is false
    assert r.slots[0] == 9 and len(r.evicted) == 0 and r.stats["collisions"] == 1
    assert t.metadata[9] == 4                               # Case 3 refreshed the home slot with new1's value
    r = t.remap([new1], 5, [1])                             # the short-lived id is gone, the long-lived stays
    assert r.slots[0] == 9 and r.evicted.tolist() == [9] and t.identities[10] == long_
    r = t.remap([new2], 12, [1])                            # 12 < 12 false: long_ still protected; new1 (6) expired
    assert r.slots[0] == 9 and r.evicted.tolist() == [9]
    r = t.remap([new1], 13, [1])                            # now long_ (12 < 13) is expired, new2 (13) is not
    assert r.slots[0] == 10 and r.evicted.tolist() == [10]
