"""mpzch_remap_noalloc -- the entry point for callers that cannot allocate -- against mpzch_remap.

Both are called through the C ABI on twin tables with the same batches; everything a remap produces
must be identical bit for bit (the evicted list as a set).  Two calls in a row share the GPU's fixed
scratch area, the second with a smaller batch, then a third again larger; sizes beyond the fixed
maximum are rejected before anything is launched."""
import numpy as np
import pytest
import torch

from paper_2602_17050_amd import binding as mp
from paper_2602_17050_amd import workloads as wl
from gpu_common import say

pytestmark = pytest.mark.gpu


def _twin(n_slots, max_probe, kind, ttl, seed, records=False):
    a = mp.MpzchTable(n_slots, max_probe, kind, ttl, seed)
    b = mp.MpzchTable(n_slots, max_probe, kind, ttl, seed, layout=mp.LAYOUT_RECORDS if records else mp.LAYOUT_SEPARATE)
    return a, b


def _call(fn, t, ids, step):
    n = ids.numel()
    out = torch.full((max(n, 1),), -7, dtype=torch.int64, device="cuda")
    ev = torch.full((max(n, 1),), -7, dtype=torch.int64, device="cuda")
    nev = torch.full((1,), -7, dtype=torch.int64, device="cuda")
    stats = torch.full((mp.STAT_COUNT,), -7, dtype=torch.int64, device="cuda")
    fn(t.handle, t.identities, t.metadata, ids, step, out[:n], ev, nev, stats)
    torch.cuda.synchronize()
    k = int(nev.item())
    return out[:n].cpu().numpy(), np.sort(ev[:k].cpu().numpy()), k, stats.cpu().numpy()


@pytest.mark.parametrize("policy", ["ttl", "lru", "ttl-records"])
def test_noalloc_equals_remap_on_consecutive_calls(policy):
    """("ttl-records": the table of the entry point under test is kept as 16-byte records, the other as two tensors.)"""
    kind = mp.EVICT_LRU if policy == "lru" else mp.EVICT_TTL
    n_slots, max_probe, ttl, seed = 60_000, 16, 2, 4711
    a, b = _twin(n_slots, max_probe, kind, ttl, seed, records=policy.endswith("records"))
    rng = np.random.Generator(np.random.Philox(key=777))
    # the first batch fills the table to load 0.9, so the later, smaller ones evict
    sizes = [54_000, 200_000, 3_000, 0, 150_000, 64]
    evictions = 0
    for step, n in enumerate(sizes):
        step *= 2
        if step == 0:
            ids_np = wl.rank_to_id(np.arange(n))
        else:
            fresh = wl.rank_to_id(rng.integers(1_000_000 * step, 1_000_000 * (step + 1), size=n // 3))
            old = wl.zipf_ids(rng, n - n // 3, 1.1, 70_000)
            ids_np = np.concatenate([fresh, old])[rng.permutation(n)].astype(np.int64)
            if n > 10:
                ids_np[5] = -3                                    # an invalid id
        ids = torch.from_numpy(np.ascontiguousarray(ids_np)).cuda()
        say("noalloc step", step, "n", n, policy)
        ref = _call(mp.mpzch_remap, a, ids, step)
        got = _call(mp.mpzch_remap_noalloc, b, ids, step)
        assert np.array_equal(got[0], ref[0]), f"out_slots differ at step {step}"
        assert got[2] == ref[2] and np.array_equal(got[1], ref[1]), f"evicted lists differ at step {step}"
        assert np.array_equal(got[3], ref[3]), (got[3], ref[3])
        assert torch.equal(a.identities, b.identities) and torch.equal(a.metadata, b.metadata)
        evictions += int(ref[3][mp.STAT_NAMES.index("evictions")])
    assert evictions > 0
    a.close()
    b.close()


def test_noalloc_rejects_batches_beyond_its_maximum():
    t = mp.MpzchTable(1000, 8, mp.EVICT_TTL, 1, 1)
    n = mp.NOALLOC_MAX_BATCH + 1
    ids = torch.zeros(n, dtype=torch.int64, device="cuda")
    out = torch.empty(n, dtype=torch.int64, device="cuda")
    nev = torch.zeros(1, dtype=torch.int64, device="cuda")
    before = t.identities.clone()
    with pytest.raises(mp.MpzchError) as e:
        mp.mpzch_remap_noalloc(t.handle, t.identities, t.metadata, ids, 1, out, out, nev, None)
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert torch.equal(before, t.identities)
    # the largest accepted batch goes through
    ids = torch.from_numpy(wl.rank_to_id(np.arange(mp.NOALLOC_MAX_BATCH) % 5000)).cuda()
    ref_t = mp.MpzchTable(1000, 8, mp.EVICT_TTL, 1, 1)
    ref = _call(mp.mpzch_remap, ref_t, ids, 1)
    got = _call(mp.mpzch_remap_noalloc, t, ids, 1)
    assert np.array_equal(got[0], ref[0]) and got[2] == ref[2] and np.array_equal(got[3], ref[3])
    assert torch.equal(ref_t.identities, t.identities) and torch.equal(ref_t.metadata, t.metadata)
    t.close()
    ref_t.close()
