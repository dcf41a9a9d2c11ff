"""Row movers and the streaming delta (Sec. 3.4 reset of weights + optimizer state, Sec. 3.7 lookup
followed by the embedding gather, Sec. 3.8 sparse delta publishing) against plain numpy statements."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_17050_amd import binding as mp
from paper_2602_17050_amd import workloads as wl
from gpu_common import Pair, say

pytestmark = pytest.mark.gpu


def test_reset_rows_multi_resets_weights_and_optimizer_state_in_one_launch():
    dev = "cuda"
    w_np = wl.embedding_pattern(1000, 64, np.float32)
    m_np = wl.embedding_pattern(1000, 1, np.float32) + 3          # row-wise momentum, 4-byte rows
    v_np = wl.embedding_pattern(500, 32, np.float32)              # a tensor with fewer rows: slot mod rows
    w, m, v = (torch.from_numpy(a).to(dev) for a in (w_np, m_np, v_np))
    v = v.to(torch.bfloat16)
    v_np = v.float().cpu().numpy()
    slots_np = np.array([3, 999, 1500, 42, 7, 100000], dtype=np.int64)
    slots = torch.from_numpy(slots_np).to(dev)
    cnt = torch.tensor([5], dtype=torch.int64, device=dev)
    init_m = torch.full((1,), 0.25, dtype=torch.float32, device=dev)
    mp.mpzch_reset_rows_multi(slots, cnt, [w, m, v], [None, init_m, None])
    torch.cuda.synchronize()
    oracle.reset_rows(slots_np[:5], w_np)
    oracle.reset_rows(slots_np[:5], m_np, np.array([0.25], np.float32))
    oracle.reset_rows(slots_np[:5], v_np)
    assert np.array_equal(w.cpu().numpy(), w_np)
    assert np.array_equal(m.cpu().numpy(), m_np)
    assert np.array_equal(v.float().cpu().numpy(), v_np)


LAYOUTS = ("separate", "records")


@pytest.mark.parametrize("layout", LAYOUTS)
def test_lookup_gather_returns_the_rows_of_the_looked_up_slots(layout):
    """One kernel resolves the slots and copies the rows (Sec. 3.7); the slots themselves are an optional output."""
    p = Pair(50_000, 16, 3, True, 77, layout=layout)
    rng = np.random.Generator(np.random.Philox(key=11))
    for step in range(4):
        p.step(wl.zipf_ids(rng, 20_000, 1.05, 60_000), step, check_state=False)
    cases = ((32, torch.float32, 20_000), (128, torch.bfloat16, 20_000), (3, torch.float32, 20_000),
             (1, torch.float32, 50_000), (40, torch.float32, 7), (256, torch.float32, 50_000))
    for k, (dim, dtype, nrows) in enumerate(cases):
        rows_np = wl.embedding_pattern(nrows, dim, np.float32)            # mostly fewer rows than slots
        rows = torch.from_numpy(rows_np).cuda().to(dtype)
        q = np.concatenate([wl.zipf_ids(rng, 5000 + 37 * k, 1.05, 60_000), rng.integers(-3, 1 << 40, size=500)])
        q = q[rng.permutation(len(q))]
        ids = torch.from_numpy(q).cuda()
        out = torch.full((len(q), dim), -1, dtype=dtype, device="cuda")
        slots = torch.empty(len(q), dtype=torch.int64, device="cuda") if k % 2 == 0 else None
        found = torch.empty(len(q), dtype=torch.uint8, device="cuda") if k % 3 != 2 else None
        say("lookup_gather", dim, dtype, nrows)
        mp.mpzch_lookup_gather(p.g.handle, p.g.identities, ids, rows, out, slots, found)
        torch.cuda.synchronize()
        so, fo = p.o.lookup(q)
        if slots is not None:
            assert np.array_equal(slots.cpu().numpy(), so)
        if found is not None:
            assert np.array_equal(found.cpu().numpy(), fo)
        want = oracle.gather_rows(so, rows.float().cpu().numpy())
        assert np.array_equal(out.float().cpu().numpy(), want)
    # rows with a stride: a view of every second column block
    wide = torch.from_numpy(wl.embedding_pattern(20_000, 64, np.float32)).cuda()
    view = wide[:, :32]
    q = wl.zipf_ids(rng, 3000, 1.05, 60_000)
    out = torch.empty((len(q), 32), dtype=torch.float32, device="cuda")
    mp.mpzch_lookup_gather(p.g.handle, p.g.identities, torch.from_numpy(q).cuda(), view, out)
    torch.cuda.synchronize()
    so, _ = p.o.lookup(q)
    assert np.array_equal(out.cpu().numpy(), oracle.gather_rows(so, wide.cpu().numpy()[:, :32]))
    p.close()


def test_lookup_gather_at_the_size_of_the_inference_configuration():
    """1 M ids against a 100 M-slot table 80 % full (max_probe 32), rows of 128 bf16 values: a sample of the
    output rows is compared with the oracle's lookup + gather; the whole output with mpzch_lookup + torch indexing."""
    n_slots, batch = 100_000_000, 1_000_000
    spec = wl.c3_spec(n_slots)
    n_res = int(0.8 * n_slots)
    g = mp.MpzchTable(n_slots, spec.max_probe, mp.EVICT_NONE, 0, spec.hash_seed, max_batch=1 << 22)
    chunk = 1 << 22
    tmp = torch.empty(chunk, dtype=torch.int64, device="cuda")
    for lo in range(0, n_res, chunk):
        hi = min(lo + chunk, n_res)
        g.remap(torch.from_numpy(wl.c3_prefill_ids(lo, hi)).cuda(), 0, tmp[: hi - lo])
    num_rows = 10_000_000
    rows = (torch.arange(num_rows * 128, dtype=torch.int32, device="cuda") % 30011).to(torch.bfloat16).view(num_rows, 128)
    q = wl.c3_batch(3, batch, n_res)
    ids = torch.from_numpy(q).cuda()
    out = torch.empty((batch, 128), dtype=torch.bfloat16, device="cuda")
    found = torch.empty(batch, dtype=torch.uint8, device="cuda")
    mp.mpzch_lookup_gather(g.handle, g.identities, ids, rows, out, None, found)
    sl, fd = g.lookup(ids)
    torch.cuda.synchronize()
    assert torch.equal(fd, found)
    assert torch.equal(out, rows[sl % num_rows])
    # the oracle on a sample of the positions, from a host copy of the identities
    o = oracle.Table(n_slots, spec.max_probe, oracle.EVICT_NONE, 0, spec.hash_seed, g.identities.cpu().numpy(),
                     np.zeros(n_slots, np.int32))
    pos = np.sort(np.random.default_rng(5).integers(0, batch, size=50_000))
    so, fo = o.lookup(q[pos])
    pos_t = torch.from_numpy(pos).cuda()
    assert np.array_equal(found[pos_t].cpu().numpy(), fo)
    assert torch.equal(out[pos_t], rows[torch.from_numpy(so % num_rows).cuda()])
    g.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_streaming_delta_brings_an_inference_copy_up_to_date(layout):
    """Train for a while, publish a full snapshot (identities + rows), train on, publish a delta of
    what was touched since: the inference copy must equal the training state wherever it matters.
    (The inference copy is a dense identities tensor whatever the layout of the training table.)"""
    spec = wl.c4_spec(1 / 2000)                                          # 250 K slots
    t = spec.table
    dim = 16
    p = Pair(t.num_slots, t.max_probe, t.ttl, True, t.hash_seed, layout=layout)
    rows = torch.from_numpy(wl.embedding_pattern(t.num_slots, dim, np.float32)).cuda()
    for lo in range(0, spec.prefill_ids, 50_000):
        p.step(wl.stream_prefill_ids(lo, min(lo + 50_000, spec.prefill_ids)), 0, check_state=False)
    step = spec.first_step
    for _ in range(3):
        p.step(wl.stream_batch(spec, step), step, check_state=False)
        step += 1
    # full snapshot: identities only (metadata is not published, Sec. 3.7) + rows
    inf_I = p.g.identities.clone()
    inf_rows = rows.clone()
    since = step
    touched_rows = []
    for _ in range(4):
        ids = wl.stream_batch(spec, step)
        r = p.step(ids, step, check_state=False)
        # "training": every row that was looked up changes, evicted rows are reset first
        p.g.reset_rows(rows)
        sl = torch.from_numpy(np.unique(r.slots)).cuda()
        rows[sl] += float(step)
        touched_rows.append(np.unique(r.slots))
        step += 1
    cap = t.num_slots
    d_slots = torch.empty(cap, dtype=torch.int64, device="cuda")
    d_ids = torch.empty(cap, dtype=torch.int64, device="cuda")
    d_cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    mp.mpzch_collect_delta(p.g.handle, p.g.identities, p.g.metadata, since, d_slots, d_ids, d_cnt)
    n = int(d_cnt.item())
    so, io = oracle.collect_delta(p.o, since)
    got = d_slots[:n].cpu().numpy()
    order = np.argsort(got)
    assert np.array_equal(got[order], so) and np.array_equal(d_ids[:n].cpu().numpy()[order], io)
    assert set(np.concatenate(touched_rows).tolist()) <= set(so.tolist())     # every touched slot is in the delta
    say("delta entries", n, "of", t.num_slots)
    payload = torch.empty((cap, dim), dtype=torch.float32, device="cuda")
    mp.mpzch_gather_rows(d_slots, d_cnt, rows, payload)
    mp.mpzch_apply_delta(inf_I, d_slots, d_ids, d_cnt, inf_rows, payload)
    torch.cuda.synchronize()
    assert torch.equal(inf_I, p.g.identities)
    assert torch.equal(inf_rows, rows)
    # truncated output: the count is still the true one
    small = torch.empty(10, dtype=torch.int64, device="cuda")
    mp.mpzch_collect_delta(p.g.handle, p.g.identities, p.g.metadata, since, small, small.clone(), d_cnt)
    assert int(d_cnt.item()) == n
    # identities-only delta
    inf2 = torch.full_like(inf_I, -1)
    mp.mpzch_apply_delta(inf2, d_slots, d_ids, torch.tensor([n], dtype=torch.int64, device="cuda"))
    torch.cuda.synchronize()
    assert torch.equal(inf2[d_slots[:n]], d_ids[:n]) and int((inf2 >= 0).sum().item()) == n
    p.close()


@pytest.mark.parametrize("layout", LAYOUTS)
def test_collect_delta_on_a_dense_multi_million_slot_table(layout):
    """Most workgroups fill their staging area many times over: every occupied slot touched since
    `since` must come out exactly once (count, slots and ids against the numpy statement)."""
    n_slots = 6_000_011
    rng = np.random.Generator(np.random.Philox(key=606))
    I = np.where(rng.random(n_slots) < 0.7, rng.integers(0, 1 << 62, size=n_slots), -1).astype(np.int64)
    M = rng.integers(0, 10, size=n_slots).astype(np.int32)
    I[1000:9000] = np.arange(8000)                                # a fully occupied, fully qualifying stretch
    M[1000:9000] = 9
    I[20000:40000] = -1                                           # and an empty one
    o = oracle.Table(n_slots, 8, oracle.EVICT_TTL, 1, 5, I, M)
    if layout == "records":
        h = mp.mpzch_create_with_layout(n_slots, 8, (mp.EVICT_TTL, 1), 5, mp.LAYOUT_RECORDS)
        rec = torch.zeros(2 * n_slots, dtype=torch.int64, device="cuda")
        gI, gM = mp.records_views(rec, n_slots)
        gI.copy_(torch.from_numpy(I).cuda())
        gM.copy_(torch.from_numpy(M).cuda())
    else:
        h = mp.mpzch_create(n_slots, 8, (mp.EVICT_TTL, 1), 5)
        gI, gM = torch.from_numpy(I).cuda(), torch.from_numpy(M).cuda()
    d_slots = torch.empty(n_slots, dtype=torch.int64, device="cuda")
    d_ids = torch.empty(n_slots, dtype=torch.int64, device="cuda")
    d_cnt = torch.zeros(1, dtype=torch.int64, device="cuda")
    for since in (0, 5, 9, 10):
        say("collect_delta since", since)
        mp.mpzch_collect_delta(h, gI, gM, since, d_slots, d_ids, d_cnt)
        n = int(d_cnt.item())
        so, io = oracle.collect_delta(o, since)
        assert n == len(so), (since, n, len(so))
        got = d_slots[:n].cpu().numpy()
        order = np.argsort(got, kind="stable")
        assert np.array_equal(got[order], so) and np.array_equal(d_ids[:n].cpu().numpy()[order], io)
    mp.mpzch_destroy(h)
