"""Keyed jagged batch over several tables in one launch sequence vs per-table oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_17050_amd import binding as mp
from paper_2602_17050_amd import workloads as wl
from gpu_common import say

pytestmark = pytest.mark.gpu


class JaggedPair:
    def __init__(self, specs, records=()):
        """records: indices of the tables kept as one tensor of 16-byte records (the others: two dense tensors)."""
        self.specs = specs
        kg = lambda e: {"lru": mp.EVICT_LRU, "expiry": mp.EVICT_TTL_EXPIRY}.get(e, mp.EVICT_TTL if e else mp.EVICT_NONE)
        ko = lambda e: {"lru": oracle.EVICT_LRU, "expiry": oracle.EVICT_TTL_EXPIRY}.get(
            e, oracle.EVICT_TTL if e else oracle.EVICT_NONE)
        self.handles = [mp.mpzch_create_with_layout(t.num_slots, t.max_probe, (kg(t.evict), t.ttl), t.hash_seed,
                                                    mp.LAYOUT_RECORDS if f in records else mp.LAYOUT_SEPARATE)
                        for f, t in enumerate(specs)]
        self.group = mp.mpzch_group_create(self.handles)
        self.I, self.M, self.rec = [], [], []
        for f, t in enumerate(specs):
            if f in records:
                self.rec.append(torch.empty(2 * t.num_slots, dtype=torch.int64, device="cuda"))
                i, m = mp.records_views(self.rec[-1], t.num_slots)
            else:
                i = torch.empty(t.num_slots, dtype=torch.int64, device="cuda")
                m = torch.empty(t.num_slots, dtype=torch.int32, device="cuda")
            self.I.append(i)
            self.M.append(m)
        for h, i, m in zip(self.handles, self.I, self.M):
            mp.mpzch_init_tensors(h, i, m)
        self.o = [oracle.Table(t.num_slots, t.max_probe, ko(t.evict), t.ttl, t.hash_seed) for t in specs]
        self.emb_o = self.emb_g = None

    def attach_rows(self, shapes):
        """shapes: per table (rows, dim) of an fp32 tensor whose rows are reset, or None."""
        self.emb_o = [None if sh is None else wl.embedding_pattern(sh[0], sh[1], np.float32) for sh in shapes]
        self.emb_g = [None if e is None else torch.from_numpy(e).cuda() for e in self.emb_o]

    def step(self, values, offsets, step, ttls=None):
        T = len(self.specs)
        v = torch.from_numpy(values).cuda()
        off = torch.from_numpy(offsets).cuda()
        out = torch.empty(len(values), dtype=torch.int64, device="cuda")
        ev_off = [int(x) for x in offsets]                  # room for every value of the feature
        ev = torch.empty(max(len(values), 1), dtype=torch.int64, device="cuda")
        nev = torch.zeros(T, dtype=torch.int64, device="cuda")
        stats = torch.zeros(T * mp.STAT_COUNT, dtype=torch.int64, device="cuda")
        if ttls is None:
            mp.mpzch_remap_jagged(self.group, self.I, self.M, v, off, step, out, ev, ev_off, nev, stats)
        else:
            mp.mpzch_remap_jagged_feature_ttl(self.group, self.I, self.M, v, torch.from_numpy(ttls).cuda(), off, step,
                                              out, ev, ev_off, nev, stats)
        torch.cuda.synchronize()
        so, evs, sts = oracle.remap_jagged(self.o, values, offsets, step, ttls)
        assert np.array_equal(out.cpu().numpy(), so)
        nev_h = nev.cpu().numpy()
        ev_h = ev.cpu().numpy()
        st_h = stats.cpu().numpy().reshape(T, mp.STAT_COUNT)
        for f in range(T):
            assert nev_h[f] == len(evs[f]), (f, nev_h[f], len(evs[f]))
            got = ev_h[ev_off[f]: ev_off[f] + nev_h[f]]
            assert np.array_equal(np.sort(got), np.sort(evs[f])), f
            assert dict(zip(mp.STAT_NAMES, st_h[f].tolist())) == sts[f], f
        if self.emb_g is not None:
            # rows of the slots that changed owner, all tables in one launch
            mp.mpzch_reset_rows_jagged(self.group, ev, ev_off, nev, self.emb_g)
            torch.cuda.synchronize()
            for f in range(T):
                if self.emb_o[f] is not None:
                    oracle.reset_rows(evs[f], self.emb_o[f])
                    assert np.array_equal(self.emb_g[f].cpu().numpy(), self.emb_o[f]), f
        return sts

    def lookup(self, values, offsets):
        """Read-only lookup of a jagged batch through the group, against per-table oracle lookups."""
        v = torch.from_numpy(values).cuda()
        off = torch.from_numpy(offsets).cuda()
        out = torch.empty(len(values), dtype=torch.int64, device="cuda")
        found = torch.empty(len(values), dtype=torch.uint8, device="cuda")
        before = [int(i.sum().item()) for i in self.I]
        mp.mpzch_lookup_jagged(self.group, self.I, v, off, out, found)
        torch.cuda.synchronize()
        so = np.empty(len(values), np.int64)
        fo = np.empty(len(values), np.uint8)
        for f, o in enumerate(self.o):
            lo, hi = int(offsets[f]), int(offsets[f + 1])
            so[lo:hi], fo[lo:hi] = o.lookup(values[lo:hi])
        assert np.array_equal(out.cpu().numpy(), so)
        assert np.array_equal(found.cpu().numpy(), fo)
        assert [int(i.sum().item()) for i in self.I] == before      # nothing written
        out2 = torch.empty(len(values), dtype=torch.int64, device="cuda")
        mp.mpzch_lookup_jagged(self.group, self.I, v, off, out2, None)
        torch.cuda.synchronize()
        assert np.array_equal(out2.cpu().numpy(), so)
        return fo

    def check_state(self):
        for f, o in enumerate(self.o):
            assert np.array_equal(self.I[f].cpu().numpy(), o.identities), f
            assert np.array_equal(self.M[f].cpu().numpy(), o.metadata), f

    def close(self):
        mp.mpzch_group_destroy(self.group)
        for h in self.handles:
            mp.mpzch_destroy(h)


def test_group_with_tables_of_both_layouts():
    """A group whose tables are kept as 16-byte records (tables 0, 2, 3) or as two dense tensors (1, 4), every
    policy among them: jagged remap, row reset, jagged lookup."""
    specs = [wl.TableSpec(700, 16, 1, True, 51), wl.TableSpec(300, 8, 1, True, 52), wl.TableSpec(900, 33, 0, "lru", 53),
             wl.TableSpec(128, 16, 1, "expiry", 54), wl.TableSpec(50, 4, 0, False, 55)]
    jp = JaggedPair(specs, records=(0, 2, 3))
    jp.attach_rows([(700, 4), (300, 8), (450, 4), None, (50, 4)])
    rng = np.random.Generator(np.random.Philox(key=6060))
    step, tot = 0, 0
    for it in range(12):
        step += int(rng.integers(0, 3))
        counts = [int(rng.integers(0, 4 * s.num_slots)) for s in specs]
        vals = [wl.rank_to_id(rng.integers(0, 5 * s.num_slots, size=c)) for s, c in zip(specs, counts)]
        values = np.concatenate(vals).astype(np.int64)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
        say("mixed-layout group step", step, counts)
        sts = jp.step(values, offsets, step, rng.integers(0, 4, size=values.size).astype(np.int32) if it % 2 else None)
        tot += sum(s["evictions"] for s in sts)
        jp.check_state()
        jp.lookup(values[::3].copy(), _offsets_of_every_third(offsets))
    assert tot > 0
    jp.close()


def _offsets_of_every_third(offsets):
    """feature offsets of values[::3] given those of values"""
    return np.array([(int(o) + 2) // 3 for o in offsets], dtype=np.int64)


def test_config5_jagged_scaled():
    """26 tables, log-uniform sizes (total capped at 2 M slots here), P = 16, TTL 5, 2 048
    samples, pooling 1..50, Zipf(1.05) ids per feature, own hash seed per table."""
    spec = wl.c5_spec(total_slots_cap=2_000_000, samples=2048)
    jp = JaggedPair(spec.tables)
    tot = dict(evictions=0, collisions=0, inserts=0, hit_pos=0)
    for step in range(1, 13):
        values, lengths, offsets = wl.c5_batch(spec, step)
        say("c5 step", step, "values", len(values))
        sts = jp.step(values, offsets, step)
        for s in sts:
            for k in tot:
                tot[k] += s[k]
    jp.check_state()
    values, lengths, offsets = wl.c5_batch(spec, 13)
    fo = jp.lookup(values, offsets)
    say("c5 lookup of an unseen batch: found fraction", float(fo.mean()))
    assert 0.3 < fo.mean() < 1.0
    say("c5 totals", tot)
    assert all(v > 0 for v in tot.values())
    jp.close()


def test_jagged_boundaries_and_empty_features():
    """Feature boundaries inside a wavefront, empty features, different P per table."""
    specs = [wl.TableSpec(50, 4, 1, True, 1), wl.TableSpec(7, 20, 0, True, 2), wl.TableSpec(300, 40, 2, False, 3),
             wl.TableSpec(1000, 9, 1, True, 4), wl.TableSpec(64, 64, 1, True, 5)]
    jp = JaggedPair(specs)
    rng = np.random.Generator(np.random.Philox(key=77))
    for step in range(10):
        counts = [int(rng.integers(0, 90)), 0 if step % 2 else int(rng.integers(0, 40)), int(rng.integers(0, 700)),
                  0 if step % 3 == 0 else int(rng.integers(0, 3000)), int(rng.integers(0, 200))]
        vals = [rng.integers(-1, 4 * s.num_slots, size=c) for s, c in zip(specs, counts)]
        values = np.concatenate(vals).astype(np.int64)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
        say("jagged step", step, counts)
        jp.step(values, offsets, step)
        jp.check_state()
        fo = jp.lookup(values, offsets)                             # the batch just remapped: mostly resident
        probe = [rng.integers(-2, 6 * s.num_slots, size=int(rng.integers(0, 500))) for s in specs]
        jp.lookup(np.concatenate(probe).astype(np.int64),
                  np.concatenate([[0], np.cumsum([len(x) for x in probe])]).astype(np.int64))
    # an entirely empty batch
    jp.step(np.empty(0, np.int64), np.zeros(len(specs) + 1, np.int64), 11)
    jp.lookup(np.empty(0, np.int64), np.zeros(len(specs) + 1, np.int64))
    jp.close()


def test_group_of_one_table_equals_plain_remap():
    spec = wl.TableSpec(500, 16, 1, True, 42)
    jp = JaggedPair([spec])
    rng = np.random.Generator(np.random.Philox(key=5))
    for step in range(6):
        values = rng.integers(0, 2000, size=1500).astype(np.int64)
        jp.step(values, np.array([0, len(values)], np.int64), step)
    jp.check_state()
    jp.close()


@pytest.mark.parametrize("kinds", [("lru",) * 4, (True, "lru", False, "expiry", "lru", True)],
                         ids=["all_lru", "mixed_policies"])
def test_jagged_group_with_every_policy(kinds):
    """Tables of different eviction policies in one group: TTL, off, LRU and expiry-step TTL
    (each table its own retention, i.e. per-feature TTL with one table per feature)."""
    shapes = [(60, 5), (300, 16), (1000, 24), (40, 40), (2000, 9), (500, 64)]
    specs = [wl.TableSpec(n, p, 1 + i % 3, k, 100 + i) for i, ((n, p), k) in enumerate(zip(shapes, kinds))]
    jp = JaggedPair(specs)
    rng = np.random.Generator(np.random.Philox(key=1234 + len(kinds)))
    tot = 0
    step = 0
    for it in range(12):
        step += int(rng.integers(0, 3))
        counts = [int(rng.integers(0, 3 * s.num_slots)) if rng.random() > 0.15 else 0 for s in specs]
        vals = [rng.integers(-1, 5 * s.num_slots, size=c) for s, c in zip(specs, counts)]
        values = np.concatenate(vals).astype(np.int64)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
        say("policies", kinds, "step", step, counts)
        sts = jp.step(values, offsets, step)
        tot += sum(s["evictions"] for s in sts)
        jp.check_state()
        for o in jp.o:
            assert o.check_state()[0] == 0
    assert tot > 0
    jp.close()


def test_jagged_regions_that_mix_features_of_different_retention():
    """Tables of the expiry-step kind whose region of the batch holds values of several features,
    each value with the retention of its feature (per-feature TTL, Sec. 3.4), next to a plain TTL
    table and an LRU table that ignore the per-value retention."""
    specs = [wl.TableSpec(400, 8, 1, "expiry", 11), wl.TableSpec(1000, 16, 2, True, 12),
             wl.TableSpec(64, 20, 0, "expiry", 13), wl.TableSpec(300, 16, 0, "lru", 14)]
    jp = JaggedPair(specs)
    rng = np.random.Generator(np.random.Philox(key=2024))
    step, tot = 0, 0
    for it in range(14):
        step += int(rng.integers(0, 3))
        counts = [int(rng.integers(0, 4 * s.num_slots)) for s in specs]
        vals = [rng.integers(0, 4 * s.num_slots, size=c) for s, c in zip(specs, counts)]
        values = np.concatenate(vals).astype(np.int64)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
        if it % 2:
            ttls = ((values >> 2) % 6).astype(np.int32)      # the id's feature decides: equal ids, equal value
        else:
            ttls = rng.integers(0, 6, size=values.size).astype(np.int32)     # copies of an id disagree
        say("feature-ttl group step", step, counts)
        sts = jp.step(values, offsets, step, ttls)
        tot += sum(s["evictions"] for s in sts)
        jp.check_state()
    assert tot > 0
    # metadata of the expiry-step tables holds step + retention, i.e. values beyond the last step
    assert int(jp.M[0].max().item()) > step and int(jp.M[2].max().item()) > step
    assert int(jp.M[1].max().item()) <= step
    jp.close()


def test_per_value_retention_needs_a_table_that_uses_it():
    specs = [wl.TableSpec(50, 4, 1, True, 1)]
    jp = JaggedPair(specs)
    values = np.arange(10, dtype=np.int64)
    with pytest.raises(mp.MpzchError):
        jp.step(values, np.array([0, 10], np.int64), 1, np.ones(10, np.int32))
    jp.close()


def test_jagged_row_reset_in_one_launch():
    """Every table of the group has its own row tensor (one has none, one has fewer rows than
    slots, one has 12-byte rows): after each jagged remap the rows of evicted slots are reset by
    ONE launch and compared with the oracle's per-table reset."""
    specs = [wl.TableSpec(200, 8, 1, True, 31), wl.TableSpec(500, 16, 1, "lru", 32), wl.TableSpec(64, 4, 0, True, 33),
             wl.TableSpec(1000, 16, 2, True, 34), wl.TableSpec(300, 8, 1, False, 35)]
    jp = JaggedPair(specs)
    jp.attach_rows([(200, 16), (500, 8), None, (256, 3), (300, 4)])
    rng = np.random.Generator(np.random.Philox(key=909))
    tot = 0
    for step in range(12):
        counts = [int(rng.integers(0, 3 * s.num_slots)) for s in specs]
        vals = [wl.rank_to_id(rng.integers(0, 6 * s.num_slots, size=c)) for s, c in zip(specs, counts)]
        values = np.concatenate(vals).astype(np.int64)
        offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
        say("jagged reset step", step, counts)
        sts = jp.step(values, offsets, step)
        tot += sum(s["evictions"] for s in sts)
    assert tot > 100
    assert sts[4]["evictions"] == 0                                   # eviction off: its rows stay as they were
    assert np.array_equal(jp.emb_o[4], wl.embedding_pattern(300, 4, np.float32))
    jp.close()
