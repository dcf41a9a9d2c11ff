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


@pytest.mark.parametrize("policy", ["ttl", "lru"])
def test_captured_step_replays_match_the_oracle(policy):
    n_slots, max_probe, ttl, seed, n, step = 50_000, 16, 2, 77, 30_000, 5
    kind_g, kind_o = (mp.EVICT_LRU, oracle.EVICT_LRU) if policy == "lru" else (mp.EVICT_TTL, oracle.EVICT_TTL)
    g = mp.MpzchTable(n_slots, max_probe, kind_g, ttl, seed, max_batch=n)
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
