"""Shared helpers of the GPU parity tests: run the same seeded batches through the HIP
library (via the C-ABI binding) and through the CPU oracle, compare bit for bit."""
import numpy as np
import torch

import oracle
from paper_2602_17050_amd import binding as mp
from paper_2602_17050_amd import workloads as wl


def say(*a):
    print(*a, flush=True)


class Pair:
    """One table on both sides."""

    def __init__(self, num_slots, max_probe, ttl, evict=True, hash_seed=0, emb=None, layout="separate",
                 fused_reset=False):
        # evict: True = TTL, False = off, "lru" = LRU, "expiry" = per-feature TTL (metadata = expiry step)
        kind_g = {"lru": mp.EVICT_LRU, "expiry": mp.EVICT_TTL_EXPIRY}.get(evict, mp.EVICT_TTL if evict else mp.EVICT_NONE)
        kind_o = {"lru": oracle.EVICT_LRU, "expiry": oracle.EVICT_TTL_EXPIRY}.get(
            evict, oracle.EVICT_TTL if evict else oracle.EVICT_NONE)
        # layout: "separate" = two dense tensors, "records" = one tensor of 16-byte records
        self.g = mp.MpzchTable(num_slots, max_probe, kind_g, ttl, hash_seed,
                               layout=mp.LAYOUT_RECORDS if layout == "records" else mp.LAYOUT_SEPARATE)
        self.o = oracle.Table(num_slots, max_probe, kind_o, ttl, hash_seed)
        self.emb_o = None
        self.emb_g = None
        # fused_reset: rows are reset by mpzch_remap_reset instead of mpzch_remap + mpzch_reset_rows
        self.fused_reset = fused_reset
        if emb is not None:                       # numpy 2-D pattern
            self.emb_o = emb.copy()
            self.emb_g = torch.from_numpy(emb).cuda()

    @classmethod
    def from_spec(cls, spec: wl.TableSpec, with_emb=True, layout="separate", fused_reset=False):
        emb = None
        if with_emb and spec.emb_rows:
            emb = wl.embedding_pattern(spec.emb_rows, spec.emb_dim, np.float32)
        return cls(spec.num_slots, spec.max_probe, spec.ttl, spec.evict, spec.hash_seed, emb, layout, fused_reset)

    def step(self, ids_np, step, check_state=True, init_row=None, ttls=None):
        ids_np = np.ascontiguousarray(ids_np, dtype=np.int64)
        ids_g = torch.from_numpy(ids_np).cuda()
        ttls_g = None if ttls is None else torch.from_numpy(np.ascontiguousarray(ttls, dtype=np.int32)).cuda()
        init_g = None if init_row is None else torch.from_numpy(init_row).cuda()
        if self.fused_reset and self.emb_g is not None and ttls is None:
            out_g = self.g.remap_reset(ids_g, step, self.emb_g, init_g)
        else:
            out_g = self.g.remap(ids_g, step, ttls=ttls_g)
            if self.emb_g is not None and ids_np.size:
                self.g.reset_rows(self.emb_g, init_g)
        torch.cuda.synchronize()
        r = self.o.remap(ids_np, step, ttls)
        if self.emb_o is not None:
            oracle.reset_rows(r.evicted, self.emb_o, init_row)
        got = out_g.cpu().numpy()
        assert np.array_equal(got, r.slots), f"out_slots differ at step {step}: {np.nonzero(got != r.slots)[0][:10]}"
        ev = self.g.evicted.cpu().numpy()
        assert len(ev) == len(r.evicted), (len(ev), len(r.evicted))
        assert np.array_equal(np.sort(ev), np.sort(r.evicted)), "evicted sets differ"
        assert len(np.unique(ev)) == len(ev)
        assert self.g.stats_dict() == r.stats, (self.g.stats_dict(), r.stats)
        if check_state:
            self.check_state()
        return r

    def check_state(self):
        I = self.g.identities.cpu().numpy()
        M = self.g.metadata.cpu().numpy()
        bad = np.nonzero(I != self.o.identities)[0]
        assert bad.size == 0, f"identities differ at {bad[:10]}: {I[bad[:10]]} vs {self.o.identities[bad[:10]]}"
        bad = np.nonzero(M != self.o.metadata)[0]
        assert bad.size == 0, f"metadata differ at {bad[:10]}"
        if self.emb_g is not None:
            assert np.array_equal(self.emb_g.cpu().numpy(), self.emb_o), "embedding rows differ"

    def lookup(self, ids_np):
        """mpzch_lookup and the counting mpzch_lookup_stats against the oracle's lookup."""
        ids_np = np.ascontiguousarray(ids_np, dtype=np.int64)
        ids_g = torch.from_numpy(ids_np).cuda()
        out, found = self.g.lookup(ids_g)
        out2 = torch.full_like(out, -9)
        found2 = torch.full_like(found, 9)
        stats = torch.full((mp.STAT_COUNT,), -9, dtype=torch.int64, device="cuda")
        mp.mpzch_lookup_stats(self.g.handle, self.g.identities, ids_g, out2, found2, stats)
        torch.cuda.synchronize()
        so, fo, st = self.o.lookup(ids_np, want_stats=True)
        assert np.array_equal(out.cpu().numpy(), so)
        assert np.array_equal(found.cpu().numpy(), fo)
        assert torch.equal(out, out2) and torch.equal(found, found2)
        got = dict(zip(mp.STAT_NAMES, stats.cpu().numpy().tolist()))
        assert got == st, (got, st)
        return so, fo

    def close(self):
        self.g.close()
