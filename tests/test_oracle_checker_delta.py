"""CPU-only pins of the oracle's helpers that the GPU tests lean on: the state checker must DETECT
each kind of broken table (planted here by hand), and the delta / gather / jagged helpers must give
hand-worked results on tiny cases (Sec. 3.6 keyed jagged batch; Sec. 3.7 gather; Sec. 3.8 sparse delta)."""
import numpy as np

import oracle
from test_oracle_pins import py_home, ids_with_home


# ---------------------------------------------------------------- oracle_check_state on planted violations
def _healthy(n=32, max_probe=4, seed=11):
    """ids with homes 5, 5, 5, 20 -> slots 5, 6, 7, 20."""
    t = oracle.Table(n, max_probe, oracle.EVICT_NONE, 0, seed)
    a, b, c = ids_with_home(5, seed, n, 3)
    d = ids_with_home(20, seed, n, 1)[0]
    r = t.remap([a, b, c, d], 1)
    assert r.slots.tolist() == [5, 6, 7, 20]
    return t, (a, b, c, d)


def test_checker_accepts_a_healthy_table():
    t, _ = _healthy()
    assert t.check_state() == (0, 4, -1)
    assert t.check_state(6, 21) == (0, 3, -1)                    # the range restricts what is examined
    assert t.check_state(8, 20) == (0, 0, -1)


def test_checker_counts_an_id_stored_twice():
    """Sec. 3.2: the two-pass design exists so that no id is ever stored in two slots."""
    t, (a, b, c, d) = _healthy()
    t.identities[8] = a                                          # a lives at 5 and again at 8 (still inside its window)
    bad, occ, first_bad = t.check_state()
    assert (bad, occ, first_bad) == (1, 5, 8)                    # a lookup of a finds slot 5, so the copy at 8 is the offender
    t.identities[4] = d                                          # and d twice, the planted copy in FRONT of nothing it could be found at
    bad, occ, first_bad = t.check_state()
    assert (bad, occ, first_bad) == (2, 6, 4)


def test_checker_counts_a_resident_outside_its_probe_range():
    """A resident must lie within min(P, N) slots of its home (Algorithm 1 probes no further)."""
    t, (a, b, c, d) = _healthy()
    t.identities[20] = -1
    t.identities[24] = d                                         # home 20, P = 4: slots 20..23 only
    assert t.check_state() == (1, 4, 24)
    assert t.check_state(0, 24) == (0, 3, -1)                    # not examined: not counted
    # before the home slot is outside as well
    t.identities[24] = -1
    t.identities[19] = d
    assert t.check_state() == (1, 4, 19)


def test_checker_counts_an_empty_slot_between_home_and_resident():
    """A slot never becomes empty again once occupied, so no empty slot may precede a resident in
    its window -- the property that lets Pass 1 stop at the first empty slot."""
    t, (a, b, c, d) = _healthy()
    t.identities[6] = -1                                         # c (home 5) sits at 7 behind a hole at 6
    assert t.check_state() == (1, 3, 7)
    t.identities[5] = -1                                         # two holes in front of c: still one offending resident
    assert t.check_state() == (1, 2, 7)


def test_checker_counts_values_that_are_neither_empty_nor_an_id():
    """Claim tags (values <= -2) must be gone when a call has finished."""
    t, _ = _healthy()
    t.identities[12] = -2
    t.identities[30] = -(1 << 62)
    bad, occ, first_bad = t.check_state()
    assert (bad, occ, first_bad) == (2, 4, 12)
    assert t.check_state(13, 32) == (1, 1, 30)


def test_checker_reports_the_first_of_several_violations_and_counts_all():
    t, (a, b, c, d) = _healthy()
    t.identities[2] = -5                                         # garbage
    t.identities[9] = b                                          # b twice (window 5..8: slot 9 is also out of range)
    t.identities[21] = -1
    t.identities[22] = ids_with_home(20, 11, 32, 2)[1]           # a new id behind a hole at 21
    bad, occ, first_bad = t.check_state()
    assert bad == 3 and first_bad == 2 and occ == 6


# ---------------------------------------------------------------- Sec. 3.8 sparse delta, Sec. 3.7 gather
def _delta_table():
    t = oracle.Table(8, 2, oracle.EVICT_TTL, 1, 0)
    t.identities[:] = [-1, 10, -1, 11, 12, -1, -1, 13]
    t.metadata[:] = [-1, 3, -1, 5, 4, 9, -1, 5]                  # slot 5 is EMPTY with a stale time stamp
    return t


def test_collect_delta_by_hand():
    """Delta = the slots that hold an id and were touched (seen, inserted or refreshed) at or after
    `since`: their metadata, the last-seen step, is >= since."""
    t = _delta_table()
    slots, ids = oracle.collect_delta(t, 5)
    assert slots.tolist() == [3, 7] and ids.tolist() == [11, 13]
    slots, ids = oracle.collect_delta(t, 4)
    assert slots.tolist() == [3, 4, 7] and ids.tolist() == [11, 12, 13]
    slots, ids = oracle.collect_delta(t, 0)
    assert slots.tolist() == [1, 3, 4, 7] and ids.tolist() == [10, 11, 12, 13]       # never an empty slot
    slots, ids = oracle.collect_delta(t, 6)
    assert slots.size == 0 and ids.size == 0
    assert slots.dtype == np.int64 and ids.dtype == np.int64


def test_collect_delta_follows_a_remap():
    seed, n = 3, 16
    x, y = ids_with_home(7, seed, n, 2)
    z = ids_with_home(1, seed, n, 1)[0]
    t = oracle.Table(n, 2, oracle.EVICT_TTL, 3, seed)
    t.remap([x, z], 1)
    t.remap([y], 2)
    t.remap([x], 4)                                              # refreshes x only
    slots, ids = oracle.collect_delta(t, 4)
    assert slots.tolist() == [7] and ids.tolist() == [x]
    slots, ids = oracle.collect_delta(t, 2)
    assert slots.tolist() == [7, 8] and ids.tolist() == [x, y]


def test_gather_rows_by_hand():
    rows = np.arange(8, dtype=np.float32).reshape(4, 2)          # row r = [2r, 2r + 1]
    got = oracle.gather_rows([1, 6, 4, 3], rows)                 # row = slot mod 4 -> 1, 2, 0, 3
    assert got.tolist() == [[2, 3], [4, 5], [0, 1], [6, 7]]
    got[0, 0] = 99
    assert rows[1, 0] == 2                                       # a copy, not a view
    assert oracle.gather_rows([], rows).shape == (0, 2)


def test_apply_delta_by_hand():
    """Sec. 3.8: a delta updates the identities entries together with the embedding rows they name."""
    ident = np.array([-1, 10, -1, 11, 12, -1, -1, 13], dtype=np.int64)
    rows = np.zeros((8, 2), dtype=np.float32)
    oracle.apply_delta(ident, [3, 6], [21, 22], rows, np.array([[1, 2], [3, 4]], dtype=np.float32))
    assert ident.tolist() == [-1, 10, -1, 21, 12, -1, 22, 13]
    assert rows.tolist() == [[0, 0]] * 3 + [[1, 2]] + [[0, 0]] * 2 + [[3, 4]] + [[0, 0]]
    # fewer rows than slots: row = slot mod rows
    small = np.zeros((4, 1), dtype=np.float32)
    oracle.apply_delta(ident, [5, 2], [31, 32], small, np.array([[7], [8]], dtype=np.float32))
    assert ident.tolist() == [-1, 10, 32, 21, 12, 31, 22, 13]
    assert small[:, 0].tolist() == [0, 7, 8, 0]
    # identities only
    oracle.apply_delta(ident, [0], [40])
    assert ident[0] == 40
    # a collected delta applied to a stale replica makes it equal to the source on the delta's slots
    t = _delta_table()
    replica = np.full(8, -1, dtype=np.int64)
    slots, ids = oracle.collect_delta(t, 0)
    oracle.apply_delta(replica, slots, ids)
    assert np.array_equal(replica, t.identities)


# ---------------------------------------------------------------- Sec. 3.6 keyed jagged batch
def test_remap_jagged_by_hand():
    """Feature f owns values[offsets[f]:offsets[f+1]] and table f; tables are independent, positions
    compare by their order inside the slice (an empty feature in the middle changes nothing)."""
    s0, s1, s2 = 101, 202, 303
    t0 = oracle.Table(8, 2, oracle.EVICT_TTL, 5, s0)
    t1 = oracle.Table(6, 2, oracle.EVICT_TTL, 5, s1)
    t2 = oracle.Table(5, 3, oracle.EVICT_TTL, 5, s2)
    # x: one VALUE that occurs in features 0 and 2; its home is slot 2 in table 0 and slot 2 in table 2
    x = next(i for i in range(10 ** 6) if py_home(i, s0, 8) == 2 and py_home(i, s2, 5) == 2)
    b, c = ids_with_home(2, s0, 8, 2, avoid=(x,))               # table 0, window 2, 3
    u, v, w = ids_with_home(4, s2, 5, 3, avoid=(x,))            # table 2, window 4, 0, 1 (wraps)
    values = [x, b, c, x, u, v, x, w]
    offsets = [0, 4, 4, 8]                                       # feature 1 is empty
    out, evs, sts = oracle.remap_jagged([t0, t1, t2], values, offsets, 1)
    # table 0: x -> 2 (round 0), b -> 3 (round 1), c finds nothing -> home 2; the second x shares slot 2
    assert out[:4].tolist() == [2, 3, 2, 2]
    assert t0.identities.tolist() == [-1, -1, x, b, -1, -1, -1, -1]
    assert sts[0]["inserts"] == 2 and sts[0]["collisions"] == 1 and sts[0]["miss_pos"] == 4
    # table 1: untouched
    assert (t1.identities == -1).all() and (t1.metadata == -1).all()
    assert sts[1]["miss_pos"] == 0 and evs[1].size == 0
    # table 2: round 0: u -> 4, x -> 2; round 1: v -> 0; round 2: w -> 1.  The x of feature 0 plays no part here.
    assert out[4:].tolist() == [4, 0, 2, 1]
    assert t2.identities.tolist() == [v, w, x, -1, u]
    assert sts[2]["inserts"] == 4 and sts[2]["hit_pos"] == 0
    assert all(e.size == 0 for e in evs)
    # next step: x is resident in both tables, each finds its own copy
    out, evs, sts = oracle.remap_jagged([t0, t1, t2], [x, x], [0, 1, 1, 2], 2)
    assert out.tolist() == [2, 2] and sts[0]["hit_pos"] == 1 and sts[2]["hit_pos"] == 1
    assert t0.metadata[2] == 2 and t2.metadata[2] == 2 and t2.metadata[4] == 1


# ---------------------------------------------------------------- the probe-length counters
def test_probe_length_counters_by_hand():
    """hit_probe_sum: slots from home up to the resident, per hit position; miss_probe_sum: slots a
    search for an absent id has to read -- up to and including the first empty slot of its range,
    or the whole range -- per miss position (the algorithmic bytes of Pass 1 are 8 x these)."""
    seed, n = 41, 16
    a, b, c, e = ids_with_home(5, seed, n, 4)
    d = ids_with_home(9, seed, n, 1)[0]
    t = oracle.Table(n, 4, oracle.EVICT_NONE, 0, seed)
    r = t.remap([a, b], 1)                                       # a -> 5, b -> 6; both searched an empty table
    assert r.slots.tolist() == [5, 6] and r.stats["miss_probe_sum"] == 1 + 1 and r.stats["hit_probe_sum"] == 0
    r = t.remap([c, d, c, b, a], 2)                              # c: 5, 6 taken, 7 empty -> 3 (twice); d: 1
    assert r.slots.tolist() == [7, 9, 7, 6, 5]
    assert r.stats["miss_probe_sum"] == 3 + 1 + 3 and r.stats["miss_pos"] == 3
    assert r.stats["hit_probe_sum"] == 2 + 1 and r.stats["hit_pos"] == 2
    f = ids_with_home(5, seed, n, 5)[4]
    r = t.remap([e], 3)                                          # 5, 6, 7 taken, 8 empty -> 4, placed at 8
    assert r.slots[0] == 8 and r.stats["miss_probe_sum"] == 4
    r = t.remap([f], 4)                                          # range 5..8 full: the whole range, then Case 3
    assert r.slots[0] == 5 and r.stats["miss_probe_sum"] == 4 and r.stats["collisions"] == 1
    # a read-only lookup counts the same way, per position, and changes nothing
    before = t.identities.copy()
    so, fo, st = t.lookup([a, f, -4, c, d + 1000003, a], want_stats=True)
    g = d + 1000003                                              # some id that is not resident
    hg = py_home(g, seed, n)
    want_len = next((k + 1 for k in range(4) if t.identities[(hg + k) % n] == -1), 4)
    assert fo.tolist() == [1, 0, 0, 1, 0, 1] and so[0] == 5 and so[1] == 5 and so[3] == 7
    assert st["hit_pos"] == 3 and st["hit_probe_sum"] == 1 + 3 + 1
    assert st["miss_pos"] == 2 and st["miss_probe_sum"] == 4 + want_len and st["invalid_pos"] == 1
    assert np.array_equal(before, t.identities)
