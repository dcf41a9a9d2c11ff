"""The launch sequence of a training step (mpzch_remap + mpzch_reset_rows) captured into a HIP
graph: once scratch is reserved the calls allocate nothing, synchronise nothing and leave their
counter block zeroed, so a captured step can be replayed.  Every replay is compared with the
oracle, with eager work and synchronisation between the replays."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_17050_amd import binding as mp
from paper_2602_17050_amd import workloads as wl
from gpu_common import say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("policy", ["ttl", "lru", "ttl-fused-records"])
def test_captured_step_replays_match_the_oracle(policy):
    """("-fused-records": the step is one mpzch_remap_reset call on a table of 16-byte records.)"""
    n_slots, max_probe, ttl, seed, n, step = 50_000, 16, 2, 77, 30_000, 5
    kind_g, kind_o = (mp.EVICT_LRU, oracle.EVICT_LRU) if policy == "lru" else (mp.EVICT_TTL, oracle.EVICT_TTL)
    fused = policy.endswith("fused-records")
    g = mp.MpzchTable(n_slots, max_probe, kind_g, ttl, seed, max_batch=n,
                      layout=mp.LAYOUT_RECORDS if fused else mp.LAYOUT_SEPARATE)
    o = oracle.Table(n_slots, max_probe, kind_o, ttl, seed)
    emb_o = wl.embedding_pattern(n_slots, 8, np.float32)
    emb_g = torch.from_numpy(emb_o).cuda()
    rng = np.random.Generator(np.random.Philox(key=4242))

    pre = wl.rank_to_id(np.arange(45_000))                       # load 0.9 at step 0: later steps evict
    g.remap(torch.from_numpy(pre).cuda(), 0)
    o.remap(pre, 0)

    ids_buf = torch.zeros(n, dtype=torch.int64, device="cuda")
    out = torch.empty(n, dtype=torch.int64, device="cuda")
    evicted = torch.empty(n, dtype=torch.int64, device="cuda")
    nev = torch.zeros(1, dtype=torch.int64, device="cuda")
    stats = torch.zeros(mp.STAT_COUNT, dtype=torch.int64, device="cuda")

    def one_step():
        if fused:
            mp.mpzch_remap_reset(g.handle, g.identities, g.metadata, ids_buf, step, out, evicted, nev, stats, emb_g)
            return
        mp.mpzch_remap(g.handle, g.identities, g.metadata, ids_buf, step, out, evicted, nev, stats)
        mp.mpzch_reset_rows(evicted, nev, emb_g)

    def check(ids, what):
        torch.cuda.synchronize()
        r = o.remap(ids, step)
        oracle.reset_rows(r.evicted, emb_o)
        assert np.array_equal(out.cpu().numpy(), r.slots), what
        k = int(nev.item())
        assert k == len(r.evicted), (what, k, len(r.evicted))
        assert np.array_equal(np.sort(evicted[:k].cpu().numpy()), np.sort(r.evicted)), what
        assert dict(zip(mp.STAT_NAMES, stats.cpu().numpy().tolist())) == r.stats, what
        assert np.array_equal(g.identities.cpu().numpy(), o.identities), what
        assert np.array_equal(g.metadata.cpu().numpy(), o.metadata), what
        assert np.array_equal(emb_g.cpu().numpy(), emb_o), what
        return r

    def batch(k):
        fresh = wl.rank_to_id(rng.integers(100_000 * (k + 1), 100_000 * (k + 2), size=n // 3))
        old = wl.zipf_ids(rng, n - n // 3, 1.1, 60_000)
        return np.concatenate([fresh, old])[rng.permutation(n)].astype(np.int64)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        b = batch(0)
        ids_buf.copy_(torch.from_numpy(b).cuda())
        one_step()                                                 # eager, before the capture
    check(b, "eager call")

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_step()
    evictions = 0
    for k in range(1, 6):
        b = batch(k)
        ids_buf.copy_(torch.from_numpy(b).cuda())                  # eager work between the replays
        say("graph replay", k, policy)
        graph.replay()
        evictions += check(b, f"replay {k}").stats["evictions"]
    assert evictions > 0
    # an eager call after the replays still starts from clean counters
    b = batch(6)
    ids_buf.copy_(torch.from_numpy(b).cuda())
    one_step()
    check(b, "eager call after the replays")
    g.close()


def test_captured_jagged_step_replays_match_the_oracle():
    """A step over a group of tables (mpzch_remap_jagged + mpzch_reset_rows_jagged) captured into a HIP
    graph after mpzch_group_reserve and one eager call (which uploads the descriptors): the replays only
    launch kernels.  Values and feature offsets live in device buffers that change between the replays;
    total_values, step and the evicted-list layout are those of the capture."""
    from test_gpu_jagged import JaggedPair

    specs = [wl.TableSpec(3000, 16, 1, True, 41), wl.TableSpec(500, 8, 1, True, 42), wl.TableSpec(2000, 40, 0, False, 43),
             wl.TableSpec(800, 16, 0, "lru", 44)]
    jp = JaggedPair(specs)
    jp.attach_rows([(3000, 8), (250, 4), None, (800, 16)])
    T, total, step = len(specs), 6000, 4
    rng = np.random.Generator(np.random.Philox(key=5150))
    mp.mpzch_group_reserve(jp.group, total)
    v = torch.zeros(total, dtype=torch.int64, device="cuda")
    off = torch.zeros(T + 1, dtype=torch.int64, device="cuda")
    out = torch.empty(total, dtype=torch.int64, device="cuda")
    ev = torch.empty(total, dtype=torch.int64, device="cuda")
    nev = torch.zeros(T, dtype=torch.int64, device="cuda")
    stats = torch.zeros(T * mp.STAT_COUNT, dtype=torch.int64, device="cuda")
    ev_off = [0, 1500, 3000, 4500, 6000]                     # fixed regions of the evicted list

    def draw(k):
        cuts = np.sort(rng.integers(0, total + 1, size=T - 1))
        offsets = np.concatenate([[0], cuts, [total]]).astype(np.int64)
        counts = np.diff(offsets)
        vals = [wl.rank_to_id(rng.integers(0, 3 * s.num_slots, size=c) + (k % 3) * s.num_slots) for s, c in zip(specs, counts)]
        return np.concatenate(vals).astype(np.int64), offsets

    def one_step(at_step=step):
        mp.mpzch_remap_jagged(jp.group, jp.I, jp.M, v, off, at_step, out, ev, ev_off, nev, stats)
        mp.mpzch_reset_rows_jagged(jp.group, ev, ev_off, nev, jp.emb_g)

    def check(values, offsets, what, at_step=step):
        torch.cuda.synchronize()
        so, evs, sts = oracle.remap_jagged(jp.o, values, offsets, at_step)
        assert np.array_equal(out.cpu().numpy(), so), what
        nev_h, ev_h = nev.cpu().numpy(), ev.cpu().numpy()
        st_h = stats.cpu().numpy().reshape(T, mp.STAT_COUNT)
        for f in range(T):
            assert nev_h[f] == len(evs[f]) <= ev_off[f + 1] - ev_off[f], (what, f)
            assert np.array_equal(np.sort(ev_h[ev_off[f]: ev_off[f] + nev_h[f]]), np.sort(evs[f])), (what, f)
            assert dict(zip(mp.STAT_NAMES, st_h[f].tolist())) == sts[f], (what, f)
            if jp.emb_o[f] is not None:
                oracle.reset_rows(evs[f], jp.emb_o[f])
                assert np.array_equal(jp.emb_g[f].cpu().numpy(), jp.emb_o[f]), (what, f)
        jp.check_state()
        return sum(s["evictions"] for s in sts)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for early in range(3):                                   # eager calls at steps 0..2 fill the tables with ids
        values, offsets = draw(early)                        # that have expired at the captured step; the first
        with torch.cuda.stream(side):                        # one uploads the descriptors of both calls
            v.copy_(torch.from_numpy(values).cuda())
            off.copy_(torch.from_numpy(offsets).cuda())
            one_step(early)
        check(values, offsets, f"eager call {early}", early)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_step()
    evictions = 0
    for k in range(1, 6):
        values, offsets = draw(k)
        v.copy_(torch.from_numpy(values).cuda())
        off.copy_(torch.from_numpy(offsets).cuda())
        say("jagged graph replay", k)
        graph.replay()
        evictions += check(values, offsets, f"replay {k}")
    assert evictions > 0
    jp.close()
