"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit
(out_slots, identities, metadata, evicted-slot set, counters, reset rows)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_17050_amd import binding as mp
from paper_2602_17050_amd import workloads as wl
from gpu_common import Pair, say

pytestmark = pytest.mark.gpu


LAYOUTS = ["separate", "records"]     # two dense tensors / one tensor of 16-byte records


@pytest.mark.parametrize("layout", LAYOUTS)
def test_config1_tiny_table_every_step(layout):
    """4 096 slots, P = 8, TTL 3, fp32 4096x16 rows, 8 Zipf(1.1) batches of 1 024 ids (then
    32 more steps so that eviction and fallback are well exercised)."""
    p = Pair.from_spec(wl.c1_spec(), layout=layout)
    tot = dict(evictions=0, collisions=0, inserts=0)
    batches = wl.c1_batches() + [(s, wl.zipf_ids(wl.rng_for(1, s), 1024, 1.1, 16384)) for s in range(9, 41)]
    for step, ids in batches:
        say("c1 step", step)
        r = p.step(ids, step)
        for k in tot:
            tot[k] += r.stats[k]
    assert tot["evictions"] > 0 and tot["inserts"] > 0
    p.close()


CASES = [
    # (slots, max_probe, ttl, evict, universe, batch, steps)
    (1, 1, 0, True, 4, 7, 6),
    (2, 5, 1, True, 6, 33, 8),
    (5, 3, 0, True, 12, 64, 10),
    (17, 8, 2, True, 60, 100, 12),
    (64, 9, 1, True, 300, 257, 12),
    (100, 16, 3, True, 500, 1000, 12),
    (100, 17, 3, False, 90, 500, 6),
    (257, 32, 2, True, 2000, 4096, 10),
    (300, 40, 1, True, 2000, 3000, 8),
    (1000, 64, 2, True, 5000, 8191, 8),
    (1000, 100, 2, True, 5000, 5000, 6),
    (2048, 200, 1, True, 9000, 6000, 6),
    (600, 600, 0, True, 3000, 2500, 6),
    (50, 1, 1, True, 200, 640, 8),
    (4099, 4, 5, True, 30000, 20000, 10),
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("case", CASES, ids=[f"N{c[0]}_P{c[1]}" for c in CASES])
def test_contended_small_tables(case, layout):
    """Small tables under heavy contention: many ids compete for few slots, windows wrap
    around the table end, P crosses every group width (8/16/32/64 and multi-chunk)."""
    n_slots, max_probe, ttl, evict, universe, batch, steps = case
    rng = np.random.Generator(np.random.Philox(key=hash(case) & 0xFFFFFFFF))
    p = Pair(n_slots, max_probe, ttl, evict, hash_seed=0xABC0 + n_slots, layout=layout)
    step = 0
    for k in range(steps):
        step += int(rng.integers(0, 3))
        kind = k % 4
        if kind == 0:
            ids = wl.zipf_ids(rng, batch, 1.1, universe)
        elif kind == 1:
            ids = rng.integers(0, universe, size=batch)                      # raw small ids
        elif kind == 2:
            ids = rng.integers(-3, universe, size=batch // 2 + 1)            # some negative ids
        else:
            ids = wl.rank_to_id(rng.integers(universe, 3 * universe, size=batch))  # mostly new ids
        say("case", case, "step", step, "n", len(ids))
        p.step(ids, step)
        bad, _, _ = p.o.check_state()
        assert bad == 0
    p.lookup(rng.integers(-2, 2 * universe, size=999))
    p.close()


def test_empty_and_single_element_batches():
    p = Pair(128, 8, 2, True, 7)
    p.step(np.empty(0, np.int64), 0)
    p.step(np.array([5]), 1)
    p.step(np.empty(0, np.int64), 2)
    p.step(np.array([5, 5, 5, -1, 6]), 3)
    p.close()


@pytest.mark.parametrize("layout,fused", [("separate", False), ("records", False), ("records", True), ("separate", True)])
def test_config2_one_million_slots(layout, fused):
    """1 M slots, P = 16, TTL 10, fp32 1Mx64 rows: prefill to load 0.3, then 50 batches of
    65 536 Zipf(1.05) ids (+5 % never-seen ids) -- insert, evict and row reset (fused: by mpzch_remap_reset)."""
    spec = wl.c2_spec()
    p = Pair.from_spec(spec, layout=layout, fused_reset=fused)
    step0, pre = wl.c2_prefill()
    p.step(pre, step0, check_state=False)
    tot_ev = 0
    for step in range(1, 51):
        r = p.step(wl.c2_batch(step), step, check_state=(step % 10 == 0))
        tot_ev += r.stats["evictions"]
        if step % 10 == 0:
            occ = int((p.o.identities >= 0).sum())
            say(f"c2 step {step}: load {occ / spec.num_slots:.3f} evictions so far {tot_ev}")
    assert tot_ev > 1000
    p.check_state()
    assert p.o.check_state()[0] == 0
    p.close()


def test_config3_lookup_scaled():
    """Read-only lookups, P = 32, table prefilled to 80 %: 95 % Zipf(1.2) over residents,
    5 % unseen ids -> home slot + found = 0.  (1/100 of the 100 M-slot table.)"""
    spec = wl.c3_spec(1_000_000)
    p = Pair(spec.num_slots, spec.max_probe, 0, False, spec.hash_seed, layout="records")
    n_res = 800_000
    for k, lo in enumerate(range(0, n_res, 100_000)):
        p.step(wl.c3_prefill_ids(lo, lo + 100_000), k, check_state=False)
    p.check_state()
    I0 = p.g.identities.clone()
    for s in range(3):
        so, fo = p.lookup(wl.c3_batch(s, 100_000, n_res))
        assert 0.93 < fo.mean() < 0.96
    assert torch.equal(I0, p.g.identities)                 # no writes
    p.close()


@pytest.mark.parametrize("fused", [False, True])
def test_config4_streaming_scaled(fused):
    """Streaming freshness at 1/500 scale: 1 M slots prefilled to 0.9, TTL 20, 10 % brand-new
    ids per step, rows addressed as slot mod rows -> sustained eviction and reset."""
    spec = wl.c4_spec(1 / 500)
    t = spec.table
    emb = wl.embedding_pattern(t.emb_rows, 32, np.float32)
    p = Pair(t.num_slots, t.max_probe, t.ttl, True, t.hash_seed, emb, fused_reset=fused)
    for lo in range(0, spec.prefill_ids, 200_000):
        p.step(wl.stream_prefill_ids(lo, min(lo + 200_000, spec.prefill_ids)), 0, check_state=False)
    p.check_state()
    tot_ev = 0
    for step in range(spec.first_step, spec.first_step + 30):
        r = p.step(wl.stream_batch(spec, step), step, check_state=(step % 10 == 0))
        tot_ev += r.stats["evictions"]
    say("c4 scaled evictions", tot_ev)
    assert tot_ev > 30 * 0.05 * spec.batch
    p.check_state()
    p.close()


@pytest.mark.parametrize("policy", ["ttl", "lru"])
def test_remap_reset_equals_remap_then_reset_rows(policy):
    """mpzch_remap_reset on small contended tables with half as many rows as slots: rows of 3 floats (4-byte
    pieces) with an init row, rows of 8 floats (16-byte pieces) set to zero, rows of 40 floats with an init row;
    and an evicted list too short for the evictions -- the fused call still resets every evicted slot's row."""
    rng = np.random.Generator(np.random.Philox(key=4242))
    evict = "lru" if policy == "lru" else True
    geoms = [(97, 3, np.float32, True), (64, 8, np.float32, False), (300, 40, np.float32, True)]
    for n_slots, dim, _, with_init in geoms:
        emb = wl.embedding_pattern(max(n_slots // 2, 1), dim, np.float32)
        p = Pair(n_slots, 8, 1, evict, 0xF00D + n_slots, emb, fused_reset=True)
        init = (np.arange(dim, dtype=np.float32) + 0.25) if with_init else None
        ev = 0
        for step in range(8):
            ids = wl.rank_to_id(rng.integers(0, 4 * n_slots, size=2 * n_slots))
            say("remap_reset", n_slots, dim, "step", step)
            ev += p.step(ids, 3 * step, init_row=init).stats["evictions"]
        assert ev > 0
        p.close()
    # a list of 4 entries for many evictions: the count is the true one and every evicted row is reset
    n_slots = 256
    g = mp.MpzchTable(n_slots, 8, mp.EVICT_TTL, 0, 5)
    o = oracle.Table(n_slots, 8, oracle.EVICT_TTL, 0, 5)
    ids0 = np.arange(n_slots, dtype=np.int64)
    g.remap(torch.from_numpy(ids0).cuda(), 0)
    o.remap(ids0, 0)
    rows = torch.ones((n_slots, 8), dtype=torch.bfloat16, device="cuda")
    out = torch.empty(n_slots, dtype=torch.int64, device="cuda")
    short = torch.full((4,), -7, dtype=torch.int64, device="cuda")
    nev = torch.zeros(1, dtype=torch.int64, device="cuda")
    ids1 = np.arange(1000, 1000 + n_slots, dtype=np.int64)
    mp.mpzch_remap_reset(g.handle, g.identities, g.metadata, torch.from_numpy(ids1).cuda(), 5, out, short, nev, None, rows)
    torch.cuda.synchronize()
    r = o.remap(ids1, 5)
    assert int(nev.item()) == len(r.evicted) > 4
    assert np.array_equal(out.cpu().numpy(), r.slots)
    want = np.ones((n_slots, 8), np.float32)
    want[r.evicted] = 0
    assert np.array_equal(rows.float().cpu().numpy(), want)
    with pytest.raises(mp.MpzchError):                                   # rows of 6 bytes
        mp.mpzch_remap_reset(g.handle, g.identities, g.metadata, torch.from_numpy(ids1).cuda(), 6, out, short, nev, None,
                             torch.zeros(4, 3, dtype=torch.bfloat16, device="cuda"))
    g.close()


def test_reset_rows_init_row_and_strides():
    """rows <- a caller-supplied init row; narrow (4-byte) and wide (16-byte) store paths."""
    dev = "cuda"
    for dim, dtype in [(16, torch.float32), (3, torch.float32), (128, torch.bfloat16), (6, torch.bfloat16)]:
        rows_np = wl.embedding_pattern(50, dim, np.float32)
        rows = torch.from_numpy(rows_np).to(dev).to(dtype)
        want = rows.clone()
        slots = torch.tensor([3, 53, 7, 49, 0, 1000], dtype=torch.int64, device=dev)
        cnt = torch.tensor([5], dtype=torch.int64, device=dev)       # the last entry is beyond the count
        init = (torch.arange(dim, device=dev, dtype=torch.float32) + 0.5).to(dtype)
        mp.mpzch_reset_rows(slots, cnt, rows, init)
        want[[3, 7, 49, 0]] = init
        assert torch.equal(rows, want)
        mp.mpzch_reset_rows(slots, cnt, rows, None)
        want[[3, 7, 49, 0]] = 0
        assert torch.equal(rows, want)
        cnt.fill_(100)                                              # count beyond capacity is clamped
        mp.mpzch_reset_rows(slots[:2], cnt, rows, init)
        want[3] = init
        assert torch.equal(rows, want)


def test_results_do_not_depend_on_scheduling():
    """Same batches twice from scratch -> identical tensors (the claim protocol has one fixed
    point whatever the interleaving of wavefronts)."""
    outs = []
    for _ in range(2):
        g = mp.MpzchTable(3000, 16, mp.EVICT_TTL, 1, 99)
        res = []
        for step in range(12):
            ids = torch.from_numpy(wl.zipf_ids(wl.rng_for(9, step), 20000, 1.05, 12000)).cuda()
            res.append(g.remap(ids, step).clone())
        torch.cuda.synchronize()
        outs.append((torch.cat(res), g.identities.clone(), g.metadata.clone()))
        g.close()
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_evicted_list_truncation_reports_true_count():
    g = mp.MpzchTable(64, 8, mp.EVICT_TTL, 0, 3)
    ids0 = torch.arange(0, 64, dtype=torch.int64, device="cuda")
    g.remap(ids0, 0)
    out = torch.empty(64, dtype=torch.int64, device="cuda")
    ev = torch.full((4,), -7, dtype=torch.int64, device="cuda")
    nev = torch.zeros(1, dtype=torch.int64, device="cuda")
    ids1 = torch.arange(1000, 1064, dtype=torch.int64, device="cuda")
    mp.mpzch_remap(g.handle, g.identities, g.metadata, ids1, 5, out, ev, nev, None)
    torch.cuda.synchronize()
    o = oracle.Table(64, 8, oracle.EVICT_TTL, 0, 3)
    o.remap(ids0.cpu().numpy(), 0)
    r = o.remap(ids1.cpu().numpy(), 5)
    assert int(nev.item()) == len(r.evicted) > 4
    assert set(ev.tolist()) <= set(r.evicted.tolist()) and len(set(ev.tolist())) == 4
    assert np.array_equal(out.cpu().numpy(), r.slots)
    g.close()


def test_bad_arguments_are_rejected_before_launch():
    g = mp.MpzchTable(64, 8, mp.EVICT_TTL, 0, 3)
    ids = torch.arange(4, dtype=torch.int64, device="cuda")
    out = torch.empty(4, dtype=torch.int64, device="cuda")
    with pytest.raises(mp.MpzchError):
        mp.mpzch_remap(g.handle, g.identities, g.metadata, ids, -1, out, out, g.num_evicted, None)   # step < 0
    with pytest.raises(mp.MpzchError):
        mp.mpzch_remap(g.handle, g.identities, None, ids, 1, out, out, g.num_evicted, None)          # no metadata
    rows = torch.zeros(4, 3, dtype=torch.bfloat16, device="cuda")                                     # 6-byte rows
    with pytest.raises(mp.MpzchError):
        mp.mpzch_reset_rows(out, g.num_evicted, rows)
    g.close()


def test_a_record_table_is_rejected_unless_its_tensors_are_one_tensor_of_aligned_records():
    """Every entry point that reads a table kept as 16-byte records checks, before anything is launched, that
    the identities start at a multiple of 16 bytes (and, where it writes metadata, that metadata is the third
    word of the same records)."""
    n = 64
    h = mp.mpzch_create_with_layout(n, 8, (mp.EVICT_TTL, 1), 3, mp.LAYOUT_RECORDS)
    rec = torch.zeros(2 * n + 2, dtype=torch.int64, device="cuda")
    good_i, good_m = mp.records_views(rec[: 2 * n], n)
    odd_i, odd_m = mp.records_views(rec[1: 2 * n + 1], n)             # 8 bytes off
    mp.mpzch_init_tensors(h, good_i, good_m)
    ids = torch.arange(4, dtype=torch.int64, device="cuda")
    out = torch.empty(4, dtype=torch.int64, device="cuda")
    nev = torch.zeros(1, dtype=torch.int64, device="cuda")
    stats = torch.zeros(mp.STAT_COUNT, dtype=torch.int64, device="cuda")
    rows = torch.zeros(n, 4, dtype=torch.float32, device="cuda")
    out_rows = torch.zeros(4, 4, dtype=torch.float32, device="cuda")
    other_m = torch.zeros(n, dtype=torch.int32, device="cuda")
    before = rec.clone()
    calls = [
        lambda: mp.mpzch_remap(h, odd_i, odd_m, ids, 1, out, out.clone(), nev, None),
        lambda: mp.mpzch_remap(h, good_i, other_m, ids, 1, out, out.clone(), nev, None),       # metadata elsewhere
        lambda: mp.mpzch_remap_noalloc(h, odd_i, odd_m, ids, 1, out, out.clone(), nev, None),
        lambda: mp.mpzch_lookup(h, odd_i, ids, out),
        lambda: mp.mpzch_lookup_stats(h, odd_i, ids, out, None, stats),
        lambda: mp.mpzch_lookup_gather(h, odd_i, ids, rows, out_rows),
        lambda: mp.mpzch_init_tensors(h, odd_i, odd_m),
    ]
    for k, call in enumerate(calls):
        with pytest.raises(mp.MpzchError) as e:
            call()
        assert e.value.status == 1, k                                  # MPZCH_ERR_INVALID_ARG
    grp = mp.mpzch_group_create([h])
    with pytest.raises(mp.MpzchError):
        mp.mpzch_lookup_jagged(grp, [odd_i], ids, torch.tensor([0, 4], dtype=torch.int64, device="cuda"), out)
    mp.mpzch_group_destroy(grp)
    torch.cuda.synchronize()
    assert torch.equal(rec, before)
    mp.mpzch_lookup(h, good_i, ids, out)                               # and the well-formed call goes through
    torch.cuda.synchronize()
    mp.mpzch_destroy(h)


def test_kernel_timing_modes_count_the_launches_they_bracket():
    """mpzch_set_kernel_timing: 1 = every kernel of every call, 2 = the Pass-1 kernel of every call, 3 = the
    Pass-1 kernel of every fourth call; mpzch_kernel_times returns what was bracketed and clears the record."""
    g = mp.MpzchTable(5000, 8, mp.EVICT_TTL, 2, 11)
    rng = np.random.Generator(np.random.Philox(key=99))
    calls = 10

    def run(mode):
        mp.mpzch_set_kernel_timing(g.handle, mode)
        for k in range(calls):
            g.remap(torch.from_numpy(rng.integers(0, 20000, size=3000)).cuda(), k)
        g.lookup(torch.from_numpy(rng.integers(0, 20000, size=3000)).cuda())
        torch.cuda.synchronize()
        t = mp.mpzch_kernel_times(g.handle)
        mp.mpzch_set_kernel_timing(g.handle, 0)
        return t

    t = run(1)
    assert {k: v[1] for k, v in t.items()} == {"k_discover": calls, "k_allocate": calls, "k_finalize": calls, "k_lookup": 1}
    assert all(v[0] > 0 for v in t.values())
    t = run(2)
    assert {k: v[1] for k, v in t.items()} == {"k_discover": calls, "k_lookup": 1}
    t = run(3)                                              # 11 Pass-1 launches: the 4th and the 8th are timed
    assert sum(v[1] for v in t.values()) == 2 and t["k_discover"][1] == 2
    assert mp.mpzch_kernel_times(g.handle) == {}             # the record was cleared
    t = run(0)
    assert t == {}
    g.close()
