"""CPU-only pins of the per-feature TTL mode (Sec. 3.4: "A TTL value is computed based on the current
training timestamp and a user-defined duration ... updated in the metadata tensor whenever an ID is
processed.  Any slot with a metadata value lower than the current timestamp is deemed expired", and
"per-feature TTL configurations for embedding tables that manage multiple distinct features")."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from test_oracle_pins import py_home, ids_with_home


class ExpiryAlg1:
    """One id at a time with expiry-step metadata (Sec. 3.4: value = now + duration of the id's
    feature; a stored value before now is expired), stated as a definition:
      hit     : the window holds the id -> that slot, refreshed;
      claim   : else the first slot of the window that is empty or expired -> the id moves in with
                its own expiry step (evicted exactly when the slot held an id);
      collide : else the home slot, refreshed (Case 3);
      refresh : the slot keeps the LATER of its stored expiry step and the new one (the reading under
                test; Algorithm 1 as printed overwrites: see the tests further down)."""

    def __init__(self, n_slots, max_probe, seed):
        self.I, self.M = [-1] * n_slots, [-1] * n_slots
        self.N, self.P, self.seed = n_slots, min(max_probe, n_slots), seed

    def lookup_one(self, id_, step, ttl):
        meta = step + ttl
        h = py_home(id_, self.seed, self.N)
        window = [(h + i) % self.N for i in range(self.P)]
        holding = [s for s in window if self.I[s] == id_]
        if holding:
            self.M[holding[0]] = max(self.M[holding[0]], meta)
            return holding[0], False
        free = [s for s in window if self.I[s] == -1 or self.M[s] < step]
        if free:
            evicted = self.I[free[0]] != -1
            self.I[free[0]], self.M[free[0]] = id_, meta
            return free[0], evicted
        self.M[h] = max(self.M[h], meta)
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


# ---------------------------------------------------------------- the refresh rule, where it differs from
# Algorithm 1 as printed ("M[slot] <- meta" on a hit, "M[h] <- meta" in Case 3: plain overwrites)
def test_case_3_short_lived_id_falls_back_onto_a_longer_lived_resident():
    """Sec. 3.4, second paragraph: per-feature TTL exists so that important features keep their
    data longer.  A resident stored by a long-lived feature sits in the home slot of a
    short-lived id that finds no slot.  As printed, Case 3 would store the short-lived id's value
    (step + 1 = 6) over the resident's 5 + 20 = 25 and the resident would be evictable from step 7 on;
    under the refresh rule the slot keeps 25."""
    seed, n = 17, 16
    keep, other, short = ids_with_home(9, seed, n, 3)
    t = oracle.Table(n, 2, oracle.EVICT_TTL_EXPIRY, 0, seed)
    r = t.remap([keep, other], 5, [20, 20])
    assert r.slots.tolist() == [9, 10] and t.metadata[9] == 25 and t.metadata[10] == 25
    r = t.remap([short], 5, [1])                                  # window 9, 10 full, nothing expired
    assert r.slots[0] == 9 and r.stats["collisions"] == 1 and len(r.evicted) == 0
    assert t.metadata[9] == 25                                    # as printed: 6
    r = t.remap([short], 8, [1])                                  # as printed, keep (6 < 8) would be evicted here
    assert r.slots[0] == 9 and r.stats["collisions"] == 1 and t.identities[9] == keep
    assert t.metadata[9] == 25
    # a fallback with a LATER expiry step does raise the stored value (the refresh of Case 3 is kept)
    r = t.remap([short], 9, [30])
    assert r.slots[0] == 9 and t.metadata[9] == 39 and t.identities[9] == keep


def test_case_3_two_fallbacks_of_different_retention_on_one_home_in_one_batch():
    """Two ids fall back to one home slot in one batch.  As printed, the value left behind is that of
    whichever is processed last (4 + 2 = 6 in one order, 4 + 7 = 11 in the other); the refresh rule
    gives 11 in either order, and never less than what the resident had."""
    seed, n = 23, 12
    res0, res1, a, b = ids_with_home(4, seed, n, 4)
    for order in ([0, 1], [1, 0]):
        t = oracle.Table(n, 2, oracle.EVICT_TTL_EXPIRY, 0, seed)
        t.remap([res0, res1], 4, [3, 3])                          # slots 4 and 5, expiry 7
        ids, ttls = [a, b], [2, 7]
        r = t.remap([ids[k] for k in order], 4, [ttls[k] for k in order])
        assert r.slots.tolist() == [4, 4] and r.stats["collisions"] == 2
        assert t.metadata[4] == 11 and t.metadata[5] == 7
        assert t.identities[4] == res0 and t.identities[5] == res1
    # both shorter than the resident's: nothing changes
    t = oracle.Table(n, 2, oracle.EVICT_TTL_EXPIRY, 0, seed)
    t.remap([res0, res1], 4, [9, 9])
    t.remap([a, b], 5, [1, 2])
    assert t.metadata[4] == 13 and t.metadata[5] == 13


def test_copies_of_one_id_with_different_retention():
    """One table serves several features (Sec. 3.4); the same id arrives through two of them in one
    batch.  Resident id: the slot ends with the latest expiry step among its stored value and the
    copies', whatever their order (as printed: the last copy's).  New id: the first occurrence claims
    with its own value, later copies can only raise it."""
    seed, n = 31, 16
    x, y = ids_with_home(3, seed, n, 2)
    for ttls in ([2, 9], [9, 2]):
        t = oracle.Table(n, 4, oracle.EVICT_TTL_EXPIRY, 0, seed)
        r = t.remap([x, x], 10, ttls)                             # new id, two copies
        assert r.slots.tolist() == [3, 3] and r.stats["inserts"] == 1 and r.stats["miss_pos"] == 2
        assert t.metadata[3] == 19
        r = t.remap([x, y, x], 11, [ttls[0], 5, ttls[1]])         # resident id, two copies; y is new
        assert r.slots.tolist() == [3, 4, 3] and r.stats["hit_pos"] == 2
        assert t.metadata[3] == 20 and t.metadata[4] == 16
        r = t.remap([x, x], 12, [1, 3])                           # both shorter than what is stored: unchanged
        assert t.metadata[3] == 20                                # as printed: 15
    # a copy that falls back (Case 3) raises the home slot's value as well
    a, b, c = ids_with_home(8, seed, n, 3)
    t = oracle.Table(n, 2, oracle.EVICT_TTL_EXPIRY, 0, seed)
    t.remap([a, b], 1, [4, 4])
    r = t.remap([c, c], 2, [1, 6])
    assert r.slots.tolist() == [8, 8] and r.stats["collisions"] == 1 and t.metadata[8] == 8


@given(st.data())
@settings(max_examples=120, deadline=None)
def test_expiry_batches_do_not_depend_on_the_order_of_copies(data):
    """Permuting the copies of each id among the positions that hold it (so first occurrences stay where they
    are as ids, only the ttl values move) leaves identities, slots and metadata unchanged."""
    n_slots = data.draw(st.integers(2, 20))
    max_probe = data.draw(st.integers(1, 6))
    seed = data.draw(st.integers(0, 999))
    steps = data.draw(st.lists(st.lists(st.tuples(st.integers(0, 25), st.integers(0, 5)), max_size=24),
                               min_size=1, max_size=6))
    perm_seed = data.draw(st.integers(0, 1 << 30))
    rng = np.random.default_rng(perm_seed)
    a = oracle.Table(n_slots, max_probe, oracle.EVICT_TTL_EXPIRY, 0, seed)
    b = oracle.Table(n_slots, max_probe, oracle.EVICT_TTL_EXPIRY, 0, seed)
    for step, batch in enumerate(steps):
        ids = np.array([x for x, _ in batch], dtype=np.int64)
        ttls = np.array([t for _, t in batch], dtype=np.int32)
        ttls_b = ttls.copy()
        for v in np.unique(ids):
            where = np.nonzero(ids == v)[0]
            # the claiming value is the first occurrence's: keep it, shuffle the rest
            rest = where[1:]
            ttls_b[rest] = ttls[rng.permutation(rest)] if rest.size else ttls_b[rest]
        ra = a.remap(ids, 2 * step, ttls)
        rb = b.remap(ids, 2 * step, ttls_b)
        assert np.array_equal(ra.slots, rb.slots) and np.array_equal(a.identities, b.identities)
        assert np.array_equal(a.metadata, b.metadata)
