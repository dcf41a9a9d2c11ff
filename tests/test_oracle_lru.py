"""CPU-only pins of the oracle's LRU policy (Sec. 3.4, last paragraph: "scans the probe range
to identify and evict the entry with the oldest timestamp").  The paper gives one sentence and
a figure that is not available, so the reading is this build's: first empty slot of the range,
else the oldest entry (ties: the earlier probe round), never an entry seen at the current step;
in a batch, contended slots go to the lower choice number, then the lower batch position."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from test_oracle_pins import py_home, ids_with_home, _enumerate_stable


class LruOneAtATime:
    """One id at a time, written out directly from the sentence above."""

    def __init__(self, n_slots, max_probe, seed):
        self.I = [-1] * n_slots
        self.M = [-1] * n_slots
        self.N, self.P, self.seed = n_slots, min(max_probe, n_slots), seed

    def lookup_one(self, id_, step):
        h = py_home(id_, self.seed, self.N)
        window = [(h + i) % self.N for i in range(self.P)]
        for s in window:
            if self.I[s] == id_:
                self.M[s] = step
                return s, False
        for s in window:
            if self.I[s] == -1:
                self.I[s], self.M[s] = id_, step
                return s, False
        cand = [(self.M[s], i) for i, s in enumerate(window) if self.M[s] != step]
        if cand:
            s = window[min(cand)[1]]
            self.I[s], self.M[s] = id_, step
            return s, True
        self.M[h] = step
        return h, False


@given(st.data())
@settings(max_examples=200, deadline=None)
def test_single_id_batches_follow_the_lru_sentence(data):
    n_slots = data.draw(st.integers(1, 20))
    max_probe = data.draw(st.integers(1, 24))
    seed = data.draw(st.integers(0, 1 << 20))
    universe = data.draw(st.integers(1, 50))
    calls = data.draw(st.lists(st.tuples(st.integers(0, universe), st.integers(0, 2)), min_size=1, max_size=80))
    ref = LruOneAtATime(n_slots, max_probe, seed)
    t = oracle.Table(n_slots, max_probe, oracle.EVICT_LRU, 0, seed)
    step = 0
    for id_, dstep in calls:
        step += dstep
        slot, evicted = ref.lookup_one(id_, step)
        r = t.remap([id_], step)
        assert r.slots[0] == slot and (len(r.evicted) == 1) == evicted
        assert t.identities.tolist() == ref.I and t.metadata.tolist() == ref.M


def test_lru_by_hand():
    seed, n = 21, 16
    a, b, c, d, e = ids_with_home(5, seed, n, 5)
    t = oracle.Table(n, 3, oracle.EVICT_LRU, 0, seed)
    assert t.remap([a], 1).slots[0] == 5
    assert t.remap([b], 2).slots[0] == 6
    assert t.remap([c], 3).slots[0] == 7              # window 5,6,7 full: a(1) b(2) c(3)
    assert t.remap([a], 4).slots[0] == 5              # a refreshed -> a(4) b(2) c(3)
    r = t.remap([d], 5)                               # no empty slot: the oldest is b
    assert r.slots[0] == 6 and r.evicted.tolist() == [6] and t.identities[6] == d
    r = t.remap([e, a], 6)                            # a is resident: refreshed first; e evicts c (3 < 5)
    assert r.slots.tolist() == [7, 5] and r.evicted.tolist() == [7]
    # everything in the window was seen at step 7 -> nothing may be evicted at step 7
    t.remap([a, d, e], 7)
    r = t.remap([b], 7)
    assert r.slots[0] == 5 and len(r.evicted) == 0 and r.stats["collisions"] == 1


@given(st.data())
@settings(max_examples=120, deadline=None)
def test_lru_batch_is_the_unique_stable_matching_under_choice_then_position(data):
    n_slots = data.draw(st.integers(2, 10))
    max_probe = data.draw(st.integers(1, 4))
    seed = data.draw(st.integers(0, 1 << 16))
    t = oracle.Table(n_slots, max_probe, oracle.EVICT_LRU, 0, seed)
    step = 0
    for _ in range(data.draw(st.integers(0, 4))):    # history with different time stamps
        step += 1
        t.remap(data.draw(st.lists(st.integers(0, 40), max_size=5)), step)
    step += data.draw(st.integers(0, 1))             # the batch may share the step of the last call
    resident0 = t.identities[t.identities >= 0].tolist()
    keep = data.draw(st.lists(st.sampled_from(resident0), max_size=3, unique=True)) if resident0 else []
    new = data.draw(st.lists(st.integers(100, 140), min_size=1, max_size=5, unique=True))
    batch = list(data.draw(st.permutations(keep + new)))
    batch += data.draw(st.lists(st.sampled_from(batch), max_size=3))
    I0, M0 = t.identities.copy(), t.metadata.copy()
    r = t.remap(batch, step)

    P = min(max_probe, n_slots)
    first_pos = {}
    for j, x in enumerate(batch):
        first_pos.setdefault(x, j)
    M1 = M0.copy()
    for x in first_pos:
        if x in set(resident0):
            M1[int(np.nonzero(I0 == x)[0][0])] = step
    prefs, prio = {}, {}
    for x, j in first_pos.items():
        if x in set(resident0):
            continue
        h = py_home(x, seed, n_slots)
        window = [(h + i) % n_slots for i in range(P)]
        order = [s for s in window if I0[s] == -1]
        order += [s for _, _, s in sorted((M1[s], i, s) for i, s in enumerate(window) if I0[s] >= 0 and M1[s] != step)]
        prefs[x] = order
        for k, s in enumerate(order):
            prio[(x, s)] = (k, j)
    stable = _enumerate_stable(prefs, prio)
    assert len(stable) == 1
    want = stable[0]
    for j, x in enumerate(batch):
        if x in set(resident0):
            assert r.slots[j] == int(np.nonzero(I0 == x)[0][0])
        elif want[x] is None:
            assert r.slots[j] == py_home(x, seed, n_slots)
        else:
            assert r.slots[j] == want[x]
    placed = {s: x for x, s in want.items() if s is not None}
    for s in range(n_slots):
        assert t.identities[s] == (placed[s] if s in placed else I0[s])
    assert sorted(r.evicted.tolist()) == sorted(s for s in placed if I0[s] != -1)
    assert t.check_state()[0] == 0


@given(st.data())
@settings(max_examples=60, deadline=None)
def test_lru_duplicates_and_invariants(data):
    n_slots = data.draw(st.integers(1, 32))
    max_probe = data.draw(st.integers(1, 8))
    seed = data.draw(st.integers(0, 99))
    steps = data.draw(st.lists(st.lists(st.integers(-2, 40), max_size=40), min_size=1, max_size=6))
    ta = oracle.Table(n_slots, max_probe, oracle.EVICT_LRU, 0, seed)
    tb = oracle.Table(n_slots, max_probe, oracle.EVICT_LRU, 0, seed)
    for step, batch in enumerate(steps):
        ra = ta.remap(batch, step)
        uniq = list(dict.fromkeys(batch))
        rb = tb.remap(uniq, step)
        lut = dict(zip(uniq, rb.slots.tolist()))
        assert ra.slots.tolist() == [lut[x] for x in batch]
        assert np.array_equal(ta.identities, tb.identities) and np.array_equal(ta.metadata, tb.metadata)
        assert ta.check_state()[0] == 0
        valid = [x for x in uniq if x >= 0]
        assert (ta.metadata[[lut[x] for x in valid]] == step).all()
