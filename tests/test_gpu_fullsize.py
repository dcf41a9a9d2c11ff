"""Parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times.  Tables are prefilled through the HIP path; the table state is then copied to
the host, checked with the oracle's state checker on sampled slot ranges (every resident id
must be found by a read-only lookup at exactly its own slot), and the following steps are
replayed by the oracle from that state and compared bit for bit."""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2602_17050_amd import binding as mp
from paper_2602_17050_amd import workloads as wl
from gpu_common import say

pytestmark = pytest.mark.gpu


def _prefill_stream(g, spec, chunk=1 << 24):
    out = torch.empty(chunk, dtype=torch.int64, device="cuda")
    for lo in range(0, spec.prefill_ids, chunk):
        hi = min(lo + chunk, spec.prefill_ids)
        ids = torch.arange(lo, hi, dtype=torch.int64, device="cuda") + wl.PREFILL_ID_BASE
        g.remap(ids, 0, out[: hi - lo])
    torch.cuda.synchronize()


def _sampled_state_check(o, rng, ranges=4, width=1_000_000):
    for _ in range(ranges):
        lo = int(rng.integers(0, max(o.num_slots - width, 1)))
        bad, occ, first_bad = o.check_state(lo, min(lo + width, o.num_slots))
        assert bad == 0, (lo, first_bad)
    # the wrap-around region
    bad, _, first_bad = o.check_state(max(o.num_slots - 100_000, 0), o.num_slots)
    assert bad == 0, first_bad
    bad, _, first_bad = o.check_state(0, min(100_000, o.num_slots))
    assert bad == 0, first_bad


def _stream_parity(spec, steps, emb_check_rows=0, lru=False, records=False, fused_reset=False):
    t = spec.table
    kind_g, kind_o = (mp.EVICT_LRU, oracle.EVICT_LRU) if lru else (mp.EVICT_TTL, oracle.EVICT_TTL)
    g = mp.MpzchTable(t.num_slots, t.max_probe, kind_g, t.ttl, t.hash_seed, max_batch=1 << 24,
                      layout=mp.LAYOUT_RECORDS if records else mp.LAYOUT_SEPARATE)
    t0 = time.time()
    _prefill_stream(g, spec)
    say(f"prefilled {spec.prefill_ids} ids in {time.time() - t0:.1f}s")
    I = np.ascontiguousarray(g.identities.cpu().numpy())
    M = np.ascontiguousarray(g.metadata.cpu().numpy())
    occ = int(np.count_nonzero(I >= 0))
    say(f"occupied {occ} of {t.num_slots} ({occ / t.num_slots:.3f})")
    # bounded probing: at load 0.9 with P = 16 some 5 % of the ids end without a slot (cf. Table 1)
    assert occ > 0.94 * spec.prefill_ids
    assert (I >= -1).all()                                     # no claim tag left behind
    o = oracle.Table(t.num_slots, t.max_probe, kind_o, t.ttl, t.hash_seed, I, M)
    _sampled_state_check(o, np.random.default_rng(1))
    emb = None
    if emb_check_rows:
        emb = torch.ones((t.emb_rows, t.emb_dim), dtype=torch.bfloat16, device="cuda")
    reset_rows = []
    for k in range(steps):
        step = spec.first_step + k
        ids = wl.stream_batch(spec, step)
        if emb is not None and fused_reset:
            out = g.remap_reset(torch.from_numpy(ids).cuda(), step, emb)          # mpzch_remap_reset
        else:
            out = g.remap(torch.from_numpy(ids).cuda(), step)
            if emb is not None:
                g.reset_rows(emb)
        torch.cuda.synchronize()
        r = o.remap(ids, step)
        assert np.array_equal(out.cpu().numpy(), r.slots), f"out_slots differ at step {step}"
        ev = g.evicted.cpu().numpy()
        assert np.array_equal(np.sort(ev), np.sort(r.evicted)), f"evicted set differs at step {step}"
        assert g.stats_dict() == r.stats, (g.stats_dict(), r.stats)
        # state at every slot this step touched, and at a random sample of untouched ones
        touched = torch.from_numpy(np.unique(r.slots)).cuda()
        assert np.array_equal(g.identities[touched].cpu().numpy(), o.identities[touched.cpu().numpy()])
        assert np.array_equal(g.metadata[touched].cpu().numpy(), o.metadata[touched.cpu().numpy()])
        reset_rows.append(r.evicted % t.emb_rows)
        say(f"step {step}: {r.stats}")
        assert r.stats["evictions"] > 0 and r.stats["hit_pos"] > 0
    # whole state, in blocks (keeps the host copy small)
    blk = 1 << 27
    for lo in range(0, t.num_slots, blk):
        hi = min(lo + blk, t.num_slots)
        assert np.array_equal(g.identities[lo:hi].cpu().numpy(), o.identities[lo:hi]), f"identities differ in [{lo},{hi})"
        assert np.array_equal(g.metadata[lo:hi].cpu().numpy(), o.metadata[lo:hi]), f"metadata differ in [{lo},{hi})"
    if emb is not None:
        rows = torch.from_numpy(np.unique(np.concatenate(reset_rows))).cuda()
        assert int((emb[rows] != 0).sum().item()) == 0               # reset rows hold the init value exactly
        zero_rows = int((emb.view(torch.int16)[:, 0] == 0).sum().item())
        assert zero_rows == rows.numel()                              # and no other row was touched
    g.close()


@pytest.mark.parametrize("layout", ["records", "separate"])
def test_headline_one_billion_slots_two_steps(layout):
    """1 B slots, P = 16, TTL 20, load 0.7, 4 M ids per step (the workload bench.py times), with the
    table as one tensor of 16-byte records (what bench.py times by default) and as two dense tensors."""
    _stream_parity(wl.headline_spec(), steps=2, records=layout == "records")


@pytest.mark.parametrize("layout", ["records", "separate", "records-fused"])
def test_config4_500m_slots_with_row_reset(layout):
    """500 M slots at load 0.9, 2 M ids per step, rows of a 100 M x 128 bf16 embedding
    addressed as slot mod rows ("-fused": reset by mpzch_remap_reset, what bench.py times)."""
    _stream_parity(wl.c4_spec(), steps=3, emb_check_rows=1, records=layout.startswith("records"),
                   fused_reset=layout.endswith("fused"))


def test_config4_500m_slots_lru():
    """The same stream under the LRU policy (16-lane groups per claimant at P = 16)."""
    _stream_parity(wl.c4_spec(), steps=2, lru=True)


@pytest.mark.parametrize("layout", ["separate", "records"])
def test_config3_100m_slots_lookup(layout):
    """100 M slots, 80 M resident ids, P = 32: 1 M lookups per batch, 95 % resident; every output of every batch
    is compared with the oracle, and a repeated call must return the same."""
    spec = wl.c3_spec()
    n_res = 80_000_000
    g = mp.MpzchTable(spec.num_slots, spec.max_probe, mp.EVICT_NONE, 0, spec.hash_seed, max_batch=1 << 23,
                      layout=mp.LAYOUT_RECORDS if layout == "records" else mp.LAYOUT_SEPARATE)
    chunk = 1 << 23
    out = torch.empty(chunk, dtype=torch.int64, device="cuda")
    collisions = 0
    for lo in range(0, n_res, chunk):
        hi = min(lo + chunk, n_res)
        g.remap(torch.from_numpy(wl.c3_prefill_ids(lo, hi)).cuda(), 0, out[: hi - lo])
        collisions += g.stats_dict()["collisions"]
    torch.cuda.synchronize()
    I = np.ascontiguousarray(g.identities.cpu().numpy())
    occ = int(np.count_nonzero(I >= 0))
    say(f"c3 prefill: occupied {occ}, collisions {collisions}")
    assert occ + collisions == n_res
    o = oracle.Table(spec.num_slots, spec.max_probe, oracle.EVICT_NONE, 0, spec.hash_seed, I,
                     np.zeros(spec.num_slots, np.int32))
    _sampled_state_check(o, np.random.default_rng(3))
    before = int(g.identities.sum().item())
    for s in range(4):
        ids = wl.c3_batch(s, 1_000_000, n_res)
        ids_g = torch.from_numpy(ids).cuda()
        sg, fg = g.lookup(ids_g)
        so, fo = o.lookup(ids)
        assert np.array_equal(sg.cpu().numpy(), so) and np.array_equal(fg.cpu().numpy(), fo)
        assert 0.93 < fo.mean() <= 0.951
        sg2, fg2 = g.lookup(ids_g)
        assert torch.equal(sg, sg2) and torch.equal(fg, fg2)
    assert int(g.identities.sum().item()) == before                  # read-only
    g.close()


def test_config5_26_tables_full_jagged_batch():
    """26 tables, slot counts log-uniform 1 K .. 1 B scaled to <= 1 B in total, 65 536 samples,
    pooling 1..50: one mpzch_remap_jagged call per step, two steps."""
    spec = wl.c5_spec()
    total = sum(t.num_slots for t in spec.tables)
    say("c5 tables:", [t.num_slots for t in spec.tables], "total", total)
    assert total <= 1_000_000_000 + 26_000
    handles = [mp.mpzch_create(t.num_slots, t.max_probe, (mp.EVICT_TTL, t.ttl), t.hash_seed) for t in spec.tables]
    group = mp.mpzch_group_create(handles)
    I = [torch.empty(t.num_slots, dtype=torch.int64, device="cuda") for t in spec.tables]
    M = [torch.empty(t.num_slots, dtype=torch.int32, device="cuda") for t in spec.tables]
    for h, i, m in zip(handles, I, M):
        mp.mpzch_init_tensors(h, i, m)
    os_ = [oracle.Table(t.num_slots, t.max_probe, oracle.EVICT_TTL, t.ttl, t.hash_seed) for t in spec.tables]
    T = len(spec.tables)
    # reset target: bf16 rows of 16 values, one per slot (32 GB in all); ones, so that a reset row shows
    emb = [torch.ones((t.num_slots, 16), dtype=torch.bfloat16, device="cuda") for t in spec.tables]
    reset_total = 0
    for step in (1, 8):                              # at step 8 what step 1 brought in has expired (TTL 5)
        values, lengths, offsets = wl.c5_batch(spec, step)
        say(f"c5 step {step}: {len(values)} values")
        v = torch.from_numpy(values).cuda()
        off = torch.from_numpy(offsets).cuda()
        out = torch.empty(len(values), dtype=torch.int64, device="cuda")
        ev = torch.empty(len(values), dtype=torch.int64, device="cuda")
        nev = torch.zeros(T, dtype=torch.int64, device="cuda")
        stats = torch.zeros(T * mp.STAT_COUNT, dtype=torch.int64, device="cuda")
        mp.mpzch_remap_jagged(group, I, M, v, off, step, out, ev, [int(x) for x in offsets], nev, stats)
        torch.cuda.synchronize()
        t0 = time.time()
        so, evs, sts = oracle.remap_jagged(os_, values, offsets, step)
        say(f"oracle {time.time() - t0:.1f}s")
        assert np.array_equal(out.cpu().numpy(), so)
        nev_h, ev_h = nev.cpu().numpy(), ev.cpu().numpy()
        st_h = stats.cpu().numpy().reshape(T, mp.STAT_COUNT)
        for f in range(T):
            assert nev_h[f] == len(evs[f])
            assert np.array_equal(np.sort(ev_h[offsets[f]: offsets[f] + nev_h[f]]), np.sort(evs[f]))
            assert dict(zip(mp.STAT_NAMES, st_h[f].tolist())) == sts[f], f
        # rows of the evicted slots of all 26 tables, one launch
        mp.mpzch_reset_rows_jagged(group, ev, [int(x) for x in offsets], nev, emb)
        torch.cuda.synchronize()
        for f in range(T):
            if len(evs[f]):
                rows = torch.from_numpy(np.unique(evs[f])).cuda()
                assert int((emb[f][rows] != 0).sum().item()) == 0, f
        reset_total += sum(len(e) for e in evs)
    say("c5 evictions (rows reset):", reset_total)
    assert reset_total > 1000
    zero_rows = sum(int((e.view(torch.int16)[:, 0] == 0).sum().item()) for e in emb)
    assert zero_rows == reset_total                   # a slot is evicted at most once per step; no other row touched
    del emb
    for f in range(T):
        assert np.array_equal(I[f].cpu().numpy(), os_[f].identities), f
        assert np.array_equal(M[f].cpu().numpy(), os_[f].metadata), f
    # inference over the same 26 tables: one read-only launch for a whole jagged batch
    values, lengths, offsets = wl.c5_batch(spec, 9)
    v = torch.from_numpy(values).cuda()
    out = torch.empty(len(values), dtype=torch.int64, device="cuda")
    found = torch.empty(len(values), dtype=torch.uint8, device="cuda")
    mp.mpzch_lookup_jagged(group, I, v, torch.from_numpy(offsets).cuda(), out, found)
    torch.cuda.synchronize()
    out_h, found_h = out.cpu().numpy(), found.cpu().numpy()
    for f in range(T):
        lo, hi = int(offsets[f]), int(offsets[f + 1])
        so, fo = os_[f].lookup(values[lo:hi])
        assert np.array_equal(out_h[lo:hi], so) and np.array_equal(found_h[lo:hi], fo), f
    say(f"c5 jagged lookup: {len(values)} values, found {found_h.mean():.3f}")
    for f in range(T):
        assert np.array_equal(I[f].cpu().numpy(), os_[f].identities), f      # read-only
    mp.mpzch_group_destroy(group)
    for h in handles:
        mp.mpzch_destroy(h)


def _table1_golden():
    import os
    golden = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_collision_rate.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                v = line.split()
                golden[int(v[0])] = dict(zip((8, 16, 32, 64, 128, 256, 512), map(float, v[3:])))
    return golden


T1_IDS, T1_BATCH = 150_000_000, 262144


@pytest.mark.parametrize("size_m,max_probe", [(150, 16), (200, 8), (200, 32), (300, 64)])
def test_table1_cells_at_full_scale(size_m, max_probe):
    """Sec. 3.3, Table 1 at the paper's own scale: 150 M distinct ids, eviction off.  The fraction
    of ids left without a slot must match the printed cell within 3 % relative or four standard
    deviations of the count; 2.0x capacity with P = 64 must print as the paper's 0.0000 %.  (The far-tail
    cell 200 M / P = 64 is replayed by the oracle below instead: textbook probing under a uniform hash
    gives 0.0292 % there, 2.4 % below the printed 0.0299 %, so a 3 % band around the printed value
    is not what a correct implementation lands in.)"""
    import math
    golden = _table1_golden()
    n_ids, batch = T1_IDS, T1_BATCH
    n_slots = size_m * 1_000_000
    h = mp.mpzch_create(n_slots, max_probe, (mp.EVICT_NONE, 0), wl.HASH_SEED_BASE)
    I = torch.empty(n_slots, dtype=torch.int64, device="cuda")
    M = torch.empty(n_slots, dtype=torch.int32, device="cuda")
    mp.mpzch_init_tensors(h, I, M)
    mp.mpzch_reserve(h, batch)
    calls = (n_ids + batch - 1) // batch
    stats = torch.zeros((calls, mp.STAT_COUNT), dtype=torch.int64, device="cuda")
    out = torch.empty(batch, dtype=torch.int64, device="cuda")
    nev = torch.zeros(1, dtype=torch.int64, device="cuda")
    for k, lo in enumerate(range(0, n_ids, batch)):
        ids = wl.distinct_ids_device(lo, min(lo + batch, n_ids), "cuda")
        mp.mpzch_remap(h, I, M, ids, k, out[: ids.numel()], None, nev, stats[k])
    torch.cuda.synchronize()
    tot = dict(zip(mp.STAT_NAMES, stats.sum(dim=0).tolist()))
    assert tot["hit_pos"] == 0 and tot["miss_pos"] == n_ids and tot["evictions"] == 0
    assert tot["inserts"] + tot["collisions"] == n_ids
    assert int((I >= 0).sum().item()) == tot["inserts"]            # every placed id owns exactly one slot
    got = 100.0 * tot["collisions"] / n_ids
    want = golden[size_m][max_probe]
    sigma = 100.0 * math.sqrt(max(want / 100.0 * n_ids, 1.0)) / n_ids
    say(f"table1 {size_m}M P={max_probe}: {got:.4f}% (paper {want:.4f}%)")
    assert abs(got - want) <= max(0.03 * want, 4 * sigma)
    if size_m == 300 and max_probe == 64:
        # the printed 0.0000 % means fewer than 75 of the 150 M ids; a uniform hash leaves a handful
        # (expected count about 1 at this load), the oracle included
        assert got < 0.00005 and tot["collisions"] < 10
    mp.mpzch_destroy(h)


class _Table1Replay:
    """State of the cell that the oracle replays call by call, kept between the parts of the test."""
    size_m, max_probe, parts = 200, 64, 6

    def __init__(self):
        self.n_slots = self.size_m * 1_000_000
        self.h = mp.mpzch_create(self.n_slots, self.max_probe, (mp.EVICT_NONE, 0), wl.HASH_SEED_BASE)
        self.I = torch.empty(self.n_slots, dtype=torch.int64, device="cuda")
        self.M = torch.empty(self.n_slots, dtype=torch.int32, device="cuda")
        mp.mpzch_init_tensors(self.h, self.I, self.M)
        mp.mpzch_reserve(self.h, T1_BATCH)
        self.o = oracle.Table(self.n_slots, self.max_probe, oracle.EVICT_NONE, 0, wl.HASH_SEED_BASE)
        self.calls = (T1_IDS + T1_BATCH - 1) // T1_BATCH
        self.next_call = 0
        self.collisions = 0
        self.failed = False

    def close(self):
        mp.mpzch_destroy(self.h)
        self.I = self.M = self.o = None


@pytest.fixture(scope="module")
def table1_replay():
    st = _Table1Replay()
    yield st
    st.close()


@pytest.mark.parametrize("part", range(_Table1Replay.parts))
def test_table1_cell_replayed_by_the_oracle(table1_replay, part):
    """Sec. 3.3, Table 1, the cell 200 M slots / P = 64 at full scale (150 M distinct ids, 262 144 per
    call, eviction off), with the oracle fed the same calls: collisions and out_slots of EVERY call are
    compared, and after the last call the whole identities and metadata tensors, bit for bit.  The 573
    calls are spread over the parts of this test (the oracle needs some 25 s per part), which share
    their state and must run in order."""
    st = table1_replay
    assert not st.failed and st.next_call == part * ((st.calls + st.parts - 1) // st.parts), "parts run in order"
    st.failed = True
    per_part = (st.calls + st.parts - 1) // st.parts
    out = torch.empty(T1_BATCH, dtype=torch.int64, device="cuda")
    nev = torch.zeros(1, dtype=torch.int64, device="cuda")
    stats = torch.zeros(mp.STAT_COUNT, dtype=torch.int64, device="cuda")
    t0 = time.time()
    for k in range(part * per_part, min((part + 1) * per_part, st.calls)):
        lo = k * T1_BATCH
        ids = wl.distinct_ids_device(lo, min(lo + T1_BATCH, T1_IDS), "cuda")
        n = ids.numel()
        mp.mpzch_remap(st.h, st.I, st.M, ids, k, out[:n], None, nev, stats)
        r = st.o.remap(ids.cpu().numpy(), k)
        got = dict(zip(mp.STAT_NAMES, stats.tolist()))
        assert got == r.stats, (k, got, r.stats)
        assert np.array_equal(out[:n].cpu().numpy(), r.slots), f"out_slots differ in call {k}"
        st.collisions += r.stats["collisions"]
        st.next_call = k + 1
    say(f"table1 replay part {part}: calls up to {st.next_call} of {st.calls}, {st.collisions} collisions so far, "
        f"{time.time() - t0:.1f}s")
    if st.next_call == st.calls:
        assert np.array_equal(st.I.cpu().numpy(), st.o.identities)
        assert np.array_equal(st.M.cpu().numpy(), st.o.metadata)
        pct = 100.0 * st.collisions / T1_IDS
        say(f"table1 200M P=64 replayed: {pct:.4f}% (paper 0.0299%)")
        assert 0.027 < pct < 0.031                                  # the printed 0.0299 % is context, the oracle is the bar
    st.failed = False


def test_maximum_batch_in_one_call():
    """MPZCH_MAX_BATCH = 2^30 positions in ONE remap call (32-bit positions, claim tags, set
    indices and segment arithmetic at their limits): 805 M distinct ids, of which the first
    268 M occur twice, 805 M positions apart, into an empty table of 1.2 B slots, P = 16.
    The oracle cannot replay 2^30 ids in seconds; it checks the resulting table (sampled slot
    ranges: every resident findable at its own slot, no empty slot before a resident) and looks
    up a sample of the ids on a host copy of the table; counters and duplicates are checked
    with identities that hold at any size."""
    n = 1 << 30
    distinct = 805_306_368                                    # 0.75 * 2^30
    num_slots, max_probe, seed = 1_200_000_000, 16, 0x5EED0099
    dev = torch.device("cuda")
    g = mp.MpzchTable(num_slots, max_probe, mp.EVICT_NONE, 0, seed)
    ids = torch.empty(n, dtype=torch.int64, device=dev)
    chunk = 1 << 26
    for lo in range(0, distinct, chunk):
        hi = min(lo + chunk, distinct)
        ids[lo:hi] = wl.distinct_ids_device(lo, hi, dev, salt=9)
    ids[distinct:] = ids[: n - distinct]
    out = torch.empty(n, dtype=torch.int64, device=dev)
    say("max batch: remap of", n, "positions")
    t0 = time.time()
    mp.mpzch_reserve(g.handle, n)
    g.remap(ids, 1, out)
    torch.cuda.synchronize()
    say(f"max batch: done in {time.time() - t0:.2f}s (scratch allocation included)")
    st = g.stats_dict()
    say("max batch:", st)
    assert st["hit_pos"] == 0 and st["invalid_pos"] == 0 and st["miss_pos"] == n
    assert st["distinct_miss"] == distinct and st["evictions"] == 0
    assert st["inserts"] + st["collisions"] == distinct
    assert 0 < st["collisions"] < 0.02 * distinct            # load 0.67 at P = 16 (cf. Table 1)
    assert int(g.num_evicted.item()) == 0
    # both copies of an id carry one slot; every slot is inside the table
    assert bool((out[distinct:] == out[: n - distinct]).all())
    assert int(out.min().item()) >= 0 and int(out.max().item()) < num_slots
    # the table: one resident per inserted id, no claim tag left, metadata = step where occupied
    occ_mask = g.identities >= 0
    assert int(occ_mask.sum().item()) == st["inserts"]
    assert int((g.identities < -1).sum().item()) == 0
    assert bool((g.metadata[occ_mask] == 1).all())
    del occ_mask
    # a read-only lookup of all 2^30 positions returns the same slots (found or home alike)
    sl, found = g.lookup(ids)
    assert bool((sl == out).all())
    n_found = int(found.sum().item())
    say("max batch: found positions", n_found)
    assert n_found >= st["inserts"]
    del sl, found
    # the oracle on a host copy of the table
    I = g.identities.cpu().numpy()
    o = oracle.Table(num_slots, max_probe, oracle.EVICT_NONE, 0, seed, I, np.zeros(num_slots, np.int32))
    _sampled_state_check(o, np.random.default_rng(11))
    rng = np.random.default_rng(12)
    pos = np.sort(rng.integers(0, n, size=2_000_000))
    pos_t = torch.from_numpy(pos).to(dev)
    so, fo = o.lookup(ids[pos_t].cpu().numpy())
    assert np.array_equal(out[pos_t].cpu().numpy(), so)
    assert fo.mean() > 0.97
    g.close()
