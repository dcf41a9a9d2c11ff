#!/usr/bin/env python3
"""Benchmark of the MPZCH remap hot path on one MI355X.

A step is one pass of the whole hot path over one batch that is already resident
in HBM: the remap (discover, allocate, finalize) and the reset of the embedding rows
of the evicted slots -- one mpzch_remap_reset call, whose finalize kernel also resets
the rows (--no-fused-reset: mpzch_remap followed by mpzch_reset_rows).  Prints ONE
JSON line.

Default workload ("headline"): a single 1 B-slot table (P = 16, TTL = 20 steps)
prefilled to load 0.7, 4 M ids per step from the streaming-freshness generator
(10 % brand-new ids per step, popularity of old ids decaying with age), rows of a
100 M x 128 bf16 embedding reset as slot mod rows.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")
# which tracked rocprofv3 summary holds the HBM traffic of a workload's dominant kernel
TRAFFIC_PROFILE = {"headline": "remap_headline_1Bslots_4Mids.txt", "headline-separate": "remap_headline_1Bslots_4Mids_two_tensors.txt",
                   "c4": "remap_c4_500Mslots_2Mids.txt", "c4-separate": "remap_c4_500Mslots_2Mids_two_tensors.txt",
                   "c5": "remap_jagged_c5_26tables.txt", "c5-separate": "remap_jagged_c5_26tables_two_tensors.txt",
                   "c3": "lookup_c3_100Mslots_1Mids.txt"}


def measured_ceilings():
    """Random-access rates (operations per second on an 8 GB array) measured on MI355X by
    paper_2602_17050_amd/memory_ceilings.bin and kept in profiles/memory_ceilings_mi355x.txt: aligned
    128-byte line reads, 4-byte stores, and "line read + 4-byte store into the same line".  The figures
    are read from that file so that they cannot drift; None when the file is missing."""
    keys = {"lines": "random aligned 128-byte lines", "stores": "random 4-byte stores (one per lane)",
            "line_store": "random line read + 4-byte store into the same line"}
    out = {k: None for k in keys}
    try:
        with open(os.path.join(PROFILES, "memory_ceilings_mi355x.txt")) as fh:
            for ln in fh:
                for k, prefix in keys.items():
                    if ln.startswith(prefix):
                        out[k] = float(ln.split("ms")[1].split("G ops/s")[0]) * 1e9
    except OSError:
        pass
    return out


def profiled_traffic(workload, kernel, scale):
    """HBM bytes per launch of `kernel` from the tracked rocprofv3 --pmc summary of this workload at full
    scale: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by what the counter reads for a copy
    kernel of known size (profiles/counter_calibration_mi355x.txt: FETCH_SIZE x 2.000, WRITE_SIZE x 1.000)."""
    name = TRAFFIC_PROFILE.get(workload)
    if name is None or scale != 1.0:
        return None
    try:
        with open(os.path.join(PROFILES, name)) as fh:
            for ln in fh:
                if ln.startswith("traffic:") and f"kernel={kernel} " in ln:
                    kv = dict(x.split("=") for x in ln.split()[1:])
                    return int((2.0 * float(kv["FETCH_SIZE_KiB"]) + 1.0 * float(kv["WRITE_SIZE_KiB"])) * 1024)
    except (OSError, KeyError, ValueError):
        pass
    return None


def roofline_entry(workload, scale, kernel, avg_ms, alg_bytes, lines_per_launch=None, stores_per_launch=None, note=None,
                   same_line=False):
    """`achieved` = algorithmic bytes per launch of the dominant kernel / its average duration (HIP events
    recorded by the library on the launch stream), against the 8 TB/s HBM peak."""
    ach = alg_bytes / (avg_ms * 1e-3) / 1e9
    traffic = profiled_traffic(workload, kernel, scale)
    r = {"bound": "hbm", "kernel": kernel, "achieved": round(ach, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(ach / HBM_PEAK_GBS, 5), "traffic": traffic, "avg_kernel_ms": round(avg_ms, 4),
         "alg_bytes_per_launch": round(alg_bytes),
         # all HBM bytes the kernel moves (useful or not) against the same peak
         "traffic_frac_of_peak": None if traffic is None else round(traffic / (avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    c = measured_ceilings()
    if lines_per_launch is not None and all(c.values()):
        # what the measured random-access ceilings allow for this launch: its line reads and its metadata
        # refreshes -- narrow stores into a tensor of their own, or (a table of records) stores into lines just
        # read, priced as "line read + store into the same line" instead of as a line read
        refresh = stores_per_launch or 0.0
        if same_line:
            floor_ms = (max(lines_per_launch - refresh, 0.0) / c["lines"] + refresh / c["line_store"]) * 1e3
        else:
            floor_ms = (lines_per_launch / c["lines"] + refresh / c["stores"]) * 1e3
        r["random_access_floor_ms"] = round(floor_ms, 4)
        r["frac_of_random_access_ceiling"] = round(floor_ms / avg_ms, 3)
    if note:
        r["note"] = note
    return r


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def host_cpu():
    """(model name, logical cores the process may use) of the host the oracle is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    return model, cores


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="headline", choices=["headline", "c4", "c3", "c1", "c2", "c5", "table1"])
    ap.add_argument("--scale", type=float, default=1.0, help="shrink slots and batch (quick checks only)")
    ap.add_argument("--cpu-steps", type=int, default=12,
                    help="steps the oracle replays for cpu_baseline (0 = skip); 12 headline steps are about 10 s of CPU work")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--all-kernel-timing", action="store_true",
                    help="bracket every kernel with events (a breakdown; costs a step some 30 us), not only Pass 1")
    ap.add_argument("--policy", default="ttl", choices=["ttl", "lru"], help="eviction policy (headline / c4 workloads)")
    ap.add_argument("--no-fused-reset", action="store_true",
                    help="headline / c4 / c1 / c2: a step is mpzch_remap + mpzch_reset_rows (two calls, four launches) instead of "
                         "mpzch_remap_reset (the rows are reset by the finalize kernel)")
    ap.add_argument("--layout", default="records", choices=["separate", "records"],
                    help="headline / c4: identities and metadata as one tensor of 16-byte records {int64 id, int32 "
                         "metadata, 4 unused bytes} (default: a hit then refreshes the line it has just read), or as "
                         "two dense tensors")
    ap.add_argument("--gather", action="store_true",
                    help="c3: time mpzch_lookup_gather (the lookup fused with the gather of 128 x bf16 rows) instead of mpzch_lookup")
    ap.add_argument("--graph", action="store_true",
                    help="c1 / c2: capture the timed steps into one HIP graph and time its replay (no launch overhead on the host)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU (a table shard and every operation on it are local to its GPU). "
            "Run with --gpus 1.")
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_17050_amd import binding as mp
    from paper_2602_17050_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    mp.load_library()

    if args.workload == "c3":
        return bench_lookup(args, np, torch, mp, wl, dev)
    if args.workload in ("c1", "c2"):
        return bench_small_table(args, np, torch, mp, wl, dev)
    if args.workload == "c5":
        return bench_jagged(args, np, torch, mp, wl, dev)
    if args.workload == "table1":
        return bench_table1(args, np, torch, mp, wl, dev)

    spec = wl.headline_spec(args.scale) if args.workload == "headline" else wl.c4_spec(args.scale)
    t = spec.table
    K, W = args.steps, args.warmup
    log(f"[bench] workload={args.workload} slots={t.num_slots} P={t.max_probe} ttl={t.ttl} batch={spec.batch} "
        f"prefill={spec.prefill_ids} emb={t.emb_rows}x{t.emb_dim} {t.emb_dtype}")

    kind = mp.EVICT_LRU if args.policy == "lru" else mp.EVICT_TTL
    g = mp.MpzchTable(t.num_slots, t.max_probe, kind, t.ttl, t.hash_seed, max_batch=max(spec.batch, 1 << 24),
                      layout=mp.LAYOUT_RECORDS if args.layout == "records" else mp.LAYOUT_SEPARATE)
    emb = torch.ones((t.emb_rows, t.emb_dim), dtype=torch.bfloat16, device=dev)

    # ---- prefill at step 0 (ids PREFILL_ID_BASE + k, generated on the device in chunks)
    t0 = time.perf_counter()
    chunk = 1 << 24
    out = torch.empty(chunk, dtype=torch.int64, device=dev)
    for lo in range(0, spec.prefill_ids, chunk):
        hi = min(lo + chunk, spec.prefill_ids)
        ids = torch.arange(lo, hi, dtype=torch.int64, device=dev) + wl.PREFILL_ID_BASE
        g.remap(ids, 0, out[: hi - lo])
    torch.cuda.synchronize()
    log(f"[bench] prefill {spec.prefill_ids} ids in {time.perf_counter() - t0:.2f}s")
    del out

    # ---- batches, resident in HBM before the timed region
    t0 = time.perf_counter()
    steps = [spec.first_step + i for i in range(W + K)]
    batches_np = [wl.stream_batch(spec, s) for s in steps]
    distinct = [int(np.unique(b).size) for b in batches_np[W:]]
    batches = [torch.from_numpy(b).to(dev) for b in batches_np]
    outs = torch.empty((W + K, spec.batch), dtype=torch.int64, device=dev)
    stats = torch.zeros((W + K, mp.STAT_COUNT), dtype=torch.int64, device=dev)
    nev = torch.zeros((W + K, 1), dtype=torch.int64, device=dev)
    evicted = torch.empty(spec.batch, dtype=torch.int64, device=dev)
    log(f"[bench] generated {W + K} batches in {time.perf_counter() - t0:.2f}s")

    ev_a = [torch.cuda.Event(enable_timing=True) for _ in range(W + K)]
    ev_b = [torch.cuda.Event(enable_timing=True) for _ in range(W + K)]

    fused = not args.no_fused_reset

    def one_step(i):
        if fused:                 # the rows are reset by the kernel that decides the evictions (k_finalize)
            mp.mpzch_remap_reset(g.handle, g.identities, g.metadata, batches[i], steps[i], outs[i], evicted, nev[i],
                                 stats[i], emb)
            return
        mp.mpzch_remap(g.handle, g.identities, g.metadata, batches[i], steps[i], outs[i], evicted, nev[i], stats[i])
        if args.all_kernel_timing:
            ev_a[i].record()      # the binding launches on torch's current stream, so these events see it
        mp.mpzch_reset_rows(evicted, nev[i], emb)
        if args.all_kernel_timing:
            ev_b[i].record()

    for i in range(W):
        one_step(i)
    torch.cuda.synchronize()

    # ---- state snapshot for the CPU baseline (taken outside the timed region)
    host_I = host_M = None
    if args.cpu_steps > 0:
        t0 = time.perf_counter()
        host_I = np.ascontiguousarray(g.identities.cpu().numpy())
        host_M = np.ascontiguousarray(g.metadata.cpu().numpy())
        log(f"[bench] copied table state to host in {time.perf_counter() - t0:.2f}s")

    # HIP events around the dominant kernel (Pass 1) of every fourth timed step (the 4th, 8th, ...),
    # recorded by the library on the stream it launches on (a pair of events costs a step some 8 us);
    # --all-kernel-timing brackets every kernel of every step
    if not args.no_kernel_timing:
        mp.mpzch_set_kernel_timing(g.handle, 1 if args.all_kernel_timing else 3)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(W, W + K):
        one_step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ktimes = {} if args.no_kernel_timing else mp.mpzch_kernel_times(g.handle)
    mp.mpzch_set_kernel_timing(g.handle, False)
    if ktimes and args.all_kernel_timing and not fused:
        ktimes["k_reset_rows"] = (sum(ev_a[i].elapsed_time(ev_b[i]) for i in range(W, W + K)), K)

    total_ids = spec.batch * K
    value = total_ids / elapsed
    st = stats[W:].cpu().numpy().astype(np.float64)
    sname = {n: i for i, n in enumerate(mp.STAT_NAMES)}
    hit_pos = st[:, sname["hit_pos"]].sum()
    miss_pos = st[:, sname["miss_pos"]].sum()
    d_miss = st[:, sname["distinct_miss"]].sum()
    probe_sum = st[:, sname["hit_probe_sum"]].sum()
    evictions = st[:, sname["evictions"]].sum()
    inserts = st[:, sname["inserts"]].sum()
    collisions = st[:, sname["collisions"]].sum()
    u_total = float(sum(distinct))
    u_hit = max(u_total - d_miss, 0.0)
    mean_probe = probe_sum / max(hit_pos, 1.0)
    P = min(t.max_probe, t.num_slots)

    # ---- roofline of the dominant kernel
    roofline = None
    mlen_sum = st[:, sname["miss_probe_sum"]].sum()
    mean_miss_len = mlen_sum / max(miss_pos, 1.0)
    if ktimes:
        dom = max(ktimes, key=lambda k: ktimes[k][0])     # k_discover (the only kernel timed unless --all-kernel-timing)
        ms_total, launches = ktimes[dom]
        avg_ms = ms_total / launches
        if dom == "k_discover":
            # algorithmic bytes of Pass 1 per launch: id in (8/position), slot out (8/hit position), per
            # distinct resident id its probe prefix 8(d+1) + a 4-byte metadata store, per distinct missed id
            # the slots up to the first empty one of its range (else the whole range), 8 bytes each
            alg = (8.0 * total_ids + 8.0 * hit_pos + u_hit * (8.0 * mean_probe + 4.0) + d_miss * 8.0 * mean_miss_len) / K
            # requests: one line read per position (plus the further lines of parked ids), one metadata store per hit position
            lines = total_ids / K + (miss_pos + max(probe_sum - hit_pos, 0) / 8.0) / K
            key = args.workload if args.layout == "records" else args.workload + "-separate"
            roofline = roofline_entry(key, args.scale, dom, avg_ms, alg, lines, hit_pos / K, same_line=args.layout == "records")
        else:
            roofline = {"bound": "hbm", "kernel": dom, "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": None, "traffic": None, "avg_kernel_ms": round(avg_ms, 4)}

    # ---- CPU baseline: the oracle replays the first timed steps from the same state
    cpu = None
    if args.cpu_steps > 0:
        import oracle
        o = oracle.Table(t.num_slots, t.max_probe, oracle.EVICT_LRU if args.policy == "lru" else oracle.EVICT_TTL,
                         t.ttl, t.hash_seed, host_I, host_M)
        n_cpu = min(args.cpu_steps, K)
        cpu_t = 0.0
        same = True
        for i in range(W, W + n_cpu):
            c0 = time.perf_counter()
            r = o.remap(batches_np[i], steps[i])
            cpu_t += time.perf_counter() - c0
            same = same and bool(np.array_equal(r.slots, outs[i].cpu().numpy()))
        model, host_cores = host_cpu()
        cpu = {"value": round(spec.batch * n_cpu / cpu_t, 1), "unit": "ids/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n_cpu} timed steps ({spec.batch} ids each) replayed from a host copy of the table state",
               "matches_gpu_out_slots": same, "host_cpu": model, "host_cores": host_cores,
               "ideal_scaling_extrapolation_not_measured": round(spec.batch * n_cpu / cpu_t * host_cores, 1)}
        log(f"[bench] oracle: {cpu['value']:.3e} ids/s on 1 core of {host_cores} ({model}); x{host_cores} = "
            f"{cpu['ideal_scaling_extrapolation_not_measured']:.3e} ids/s (ideal-scaling extrapolation, not measured); "
            f"out_slots identical to GPU: {same}")

    result = {
        "metric": "remapped IDs/sec (train insert+evict) at 1 GPU",
        "value": round(value, 1),
        "unit": "ids/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(elapsed / K * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int64",
        "data": "synthetic",
        "config": {
            "workload": f"{args.workload}: {t.num_slots}-slot table, P={t.max_probe}, "
                        f"{'LRU' if args.policy == 'lru' else 'TTL=' + str(t.ttl)}, load "
                        f"{spec.prefill_ids / t.num_slots:.2f}, {spec.batch} ids/step, "
                        f"{int(spec.new_fraction * 100)}% new ids/step, reset rows of {t.emb_rows}x{t.emb_dim} bf16, "
                        f"identities+metadata as {'16-byte records' if args.layout == 'records' else 'two tensors'}, "
                        f"{'one mpzch_remap_reset call' if fused else 'mpzch_remap + mpzch_reset_rows'} per step",
            "num_slots": t.num_slots, "max_probe": t.max_probe, "ttl": t.ttl, "batch": spec.batch, "scale": args.scale,
            "layout": args.layout,
        },
        "per_step": {
            "distinct_ids": round(u_total / K, 1), "hit_positions": round(hit_pos / K, 1),
            "miss_positions": round(miss_pos / K, 1), "distinct_misses": round(d_miss / K, 1),
            "inserts": round(inserts / K, 1), "evictions": round(evictions / K, 1),
            "collisions": round(collisions / K, 1), "mean_hit_probe_len": round(mean_probe, 3),
            "mean_miss_probe_len": round(mean_miss_len, 3),
        },
        "kernel_ms_per_step": kernel_ms_per_step(ktimes, K),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)


def bench_lookup(args, np, torch, mp, wl, dev):
    """Config 3: read-only lookups on a table prefilled to 80 % (P = 32)."""
    n_slots = int(100_000_000 * args.scale)
    spec = wl.c3_spec(n_slots)
    n_res = int(0.8 * n_slots)
    batch = max(int(1_000_000 * args.scale), 64)
    K, W = args.steps, args.warmup
    g = mp.MpzchTable(n_slots, spec.max_probe, mp.EVICT_NONE, 0, spec.hash_seed, max_batch=1 << 22)
    chunk = 1 << 22
    out = torch.empty(chunk, dtype=torch.int64, device=dev)
    for k, lo in enumerate(range(0, n_res, chunk)):
        hi = min(lo + chunk, n_res)
        ids = torch.from_numpy(wl.c3_prefill_ids(lo, hi)).to(dev)
        g.remap(ids, 0, out[: hi - lo])
    torch.cuda.synchronize()
    batches_np = [wl.c3_batch(s, batch, n_res) for s in range(W + K)]
    batches = [torch.from_numpy(b).to(dev) for b in batches_np]
    outs = torch.empty((W + K, batch), dtype=torch.int64, device=dev)
    found = torch.empty((W + K, batch), dtype=torch.uint8, device=dev)
    rows = out_rows = None
    if args.gather:
        # rows of 128 bf16 values, one per slot (25.6 GB at full scale); the output of a batch is 256 MB
        rows = torch.ones((n_slots, 128), dtype=torch.bfloat16, device=dev)
        out_rows = torch.empty((batch, 128), dtype=torch.bfloat16, device=dev)

    def one(i):
        if args.gather:
            mp.mpzch_lookup_gather(g.handle, g.identities, batches[i], rows, out_rows, outs[i], found[i])
        else:
            mp.mpzch_lookup(g.handle, g.identities, batches[i], outs[i], found[i])

    for i in range(W):
        one(i)
    torch.cuda.synchronize()
    mp.mpzch_set_kernel_timing(g.handle, 1 if args.all_kernel_timing else 3)
    t0 = time.perf_counter()
    for i in range(W, W + K):
        one(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ktimes = mp.mpzch_kernel_times(g.handle)
    cpu = None
    if args.cpu_steps > 0:
        import oracle
        o = oracle.Table(n_slots, spec.max_probe, oracle.EVICT_NONE, 0, spec.hash_seed,
                         g.identities.cpu().numpy(), np.zeros(n_slots, np.int32))
        c0 = time.perf_counter()
        same = True
        n_cpu = min(args.cpu_steps, K)
        for i in range(W, W + n_cpu):
            so, fo = o.lookup(batches_np[i])
            same = same and bool(np.array_equal(so, outs[i].cpu().numpy()))
        cpu_t = time.perf_counter() - c0
        cpu = {"value": round(batch * n_cpu / cpu_t, 1), "unit": "ids/s", "cores": 1, "kind": "oracle",
               "sample": f"first {n_cpu} timed batches of {batch} ids", "matches_gpu_out_slots": same}
    ms_total, launches = ktimes["k_lookup"]
    hit_frac = float(found[W:].float().mean().item())
    # byte accounting (outside the timed region): the counting lookup gives the probe lengths of the
    # timed batches, the host the number of distinct resident / absent ids
    mp.mpzch_set_kernel_timing(g.handle, 0)
    st = torch.zeros((K, mp.STAT_COUNT), dtype=torch.int64, device=dev)
    tmp_s = torch.empty(batch, dtype=torch.int64, device=dev)
    tmp_f = torch.empty(batch, dtype=torch.uint8, device=dev)
    for i in range(W, W + K):
        mp.mpzch_lookup_stats(g.handle, g.identities, batches[i], tmp_s, tmp_f, st[i - W])
    torch.cuda.synchronize()
    stn = st.cpu().numpy().astype(np.float64).sum(axis=0)
    sname = {n: i for i, n in enumerate(mp.STAT_NAMES)}
    hit_pos, miss_pos = stn[sname["hit_pos"]], stn[sname["miss_pos"]]
    mean_probe = stn[sname["hit_probe_sum"]] / max(hit_pos, 1.0)
    mean_miss_len = stn[sname["miss_probe_sum"]] / max(miss_pos, 1.0)
    u_hit = u_miss = 0.0
    for i in range(W, W + K):
        f_np = found[i].cpu().numpy().astype(bool)
        valid = batches_np[i] >= 0
        u_hit += np.unique(batches_np[i][f_np]).size
        u_miss += np.unique(batches_np[i][~f_np & valid]).size
    # per position: id in (8), slot out (8), found flag (1); per distinct resident id its probe prefix,
    # per distinct absent id the slots up to the first empty one of its range
    alg = (17.0 * batch * K + u_hit * 8.0 * mean_probe + u_miss * 8.0 * mean_miss_len) / K
    lines = batch + (miss_pos + max(stn[sname["hit_probe_sum"]] - hit_pos, 0) / 8.0) / K
    if args.gather:
        alg += 2.0 * 256.0 * batch          # every position's row read and written (256 bytes)
        lines += 2.0 * batch                # a row is two 128-byte lines
    roofline = roofline_entry("c3-gather" if args.gather else "c3", args.scale, "k_lookup", ms_total / launches, alg, lines, 0.0)
    roofline["hit_fraction"] = round(hit_frac, 4)
    result = {
        "metric": "remapped IDs/sec (infer lookup) at 1 GPU", "value": round(batch * K / elapsed, 1), "unit": "ids/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(elapsed / K * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"c3: lookup-only, {n_slots}-slot table 80% full, P=32, {batch} ids/batch, "
                               f"95% resident Zipf(1.2), 5% unseen" +
                               (", fused with the gather of 128 x bf16 rows (mpzch_lookup_gather)" if args.gather else ""),
                   "scale": args.scale},
        "per_step": {"distinct_resident_ids": round(u_hit / K, 1), "distinct_absent_ids": round(u_miss / K, 1),
                     "mean_hit_probe_len": round(mean_probe, 3), "mean_miss_probe_len": round(mean_miss_len, 3)},
        "kernel_ms_per_step": kernel_ms_per_step(ktimes, K),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)


def training_alg_bytes(np, positions, st_rows, distinct, names):
    """Algorithmic bytes of Pass 1 over some calls on ONE table: st_rows = their counter rows (float array
    [calls, STAT_COUNT]), positions = input positions in all, distinct = distinct valid ids in all.  Also
    returns the random requests (line reads, metadata stores) these calls need at least."""
    n = {k: i for i, k in enumerate(names)}
    tot = st_rows.sum(axis=0)
    hit_pos, miss_pos, d_miss = tot[n["hit_pos"]], tot[n["miss_pos"]], tot[n["distinct_miss"]]
    mean_probe = tot[n["hit_probe_sum"]] / max(hit_pos, 1.0)
    mean_miss_len = tot[n["miss_probe_sum"]] / max(miss_pos, 1.0)
    u_hit = max(distinct - d_miss, 0.0)
    alg = 8.0 * positions + 8.0 * hit_pos + u_hit * (8.0 * mean_probe + 4.0) + d_miss * 8.0 * mean_miss_len
    lines = positions + miss_pos + max(tot[n["hit_probe_sum"]] - hit_pos, 0) / 8.0
    return alg, lines, hit_pos


def kernel_ms_per_step(ktimes, K):
    """Milliseconds per step of every timed kernel; the steps that were timed are those whose Pass-1 kernel was
    (all K of them, or a sample)."""
    timed = K
    for name in ("k_discover", "k_lookup"):
        if name in ktimes:
            timed = ktimes[name][1]
    return {k: round(v[0] / max(timed, 1), 4) for k, v in ktimes.items()}


def _emit(metric, value, K, W, elapsed, workload, ktimes, cpu, extra=None, roofline=None):
    dom = max(ktimes, key=lambda k: ktimes[k][0]) if ktimes else None
    result = {
        "metric": metric, "value": round(value, 1), "unit": "ids/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(elapsed / K * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64", "data": "synthetic", "config": {"workload": workload},
        "kernel_ms_per_step": kernel_ms_per_step(ktimes, K),
        "roofline": roofline or {"bound": "hbm", "kernel": dom, "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": None, "traffic": None,
                                 "avg_kernel_ms": round(ktimes[dom][0] / ktimes[dom][1], 4) if dom else None},
        "cpu_baseline": cpu,
    }
    if extra:
        result.update(extra)
    print(json.dumps(result), flush=True)


def bench_small_table(args, np, torch, mp, wl, dev):
    """Configs 1 and 2: tables that live in L2 / Infinity Cache; every step is launch-bound."""
    if args.workload == "c1":
        spec, batches_np = wl.c1_spec(), [(s, b) for s, b in wl.c1_batches()]
        name = "c1: 4096 slots, P=8, TTL=3, 8 batches of 1024 Zipf(1.1) ids, fp32 4096x16 rows"
        W = 0
    else:
        spec = wl.c2_spec()
        batches_np = [wl.c2_prefill()] + [(s, wl.c2_batch(s)) for s in range(1, 51)]
        name = "c2: 1M slots, P=16, TTL=10, prefill 0.3 then 50 batches of 65536 Zipf(1.05) ids, fp32 1Mx64 rows"
        W = 1                                                    # the prefill call is not timed
    g = mp.MpzchTable(spec.num_slots, spec.max_probe, mp.EVICT_TTL, spec.ttl, spec.hash_seed, max_batch=1 << 19)
    emb = torch.ones((spec.emb_rows, spec.emb_dim), dtype=torch.float32, device=dev)
    batches = [(s, torch.from_numpy(b).to(dev)) for s, b in batches_np]
    outs = [torch.empty(b.numel(), dtype=torch.int64, device=dev) for _, b in batches]
    # one untimed pass on a scratch table warms the code paths; the timed pass starts from an empty table
    g2 = mp.MpzchTable(spec.num_slots, spec.max_probe, mp.EVICT_TTL, spec.ttl, spec.hash_seed, max_batch=1 << 19)
    for (s, b), o in zip(batches, outs):
        g2.remap(b, s, o)
        g2.reset_rows(emb)
    torch.cuda.synchronize()
    g2.close()
    for (s, b), o in list(zip(batches, outs))[:W]:
        g.remap(b, s, o)
    torch.cuda.synchronize()
    nb = len(batches)
    stats = torch.zeros((nb, mp.STAT_COUNT), dtype=torch.int64, device=dev)
    ev = torch.empty(max(b.numel() for _, b in batches), dtype=torch.int64, device=dev)
    nev = torch.zeros(1, dtype=torch.int64, device=dev)

    def one(i):
        s_, b_ = batches[i]
        if args.no_fused_reset:
            mp.mpzch_remap(g.handle, g.identities, g.metadata, b_, s_, outs[i], ev, nev, stats[i])
            mp.mpzch_reset_rows(ev, nev, emb)
        else:
            mp.mpzch_remap_reset(g.handle, g.identities, g.metadata, b_, s_, outs[i], ev, nev, stats[i], emb)

    if args.graph:
        # the timed steps as one captured graph: the table state before the capture is restored before the
        # timed replay (a capture only records, but the warm-up replay below runs the steps once)
        I0, M0 = g.identities.clone(), g.metadata.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(W, nb):
                one(i)
        graph.replay()
        torch.cuda.synchronize()
        g.identities.copy_(I0)
        g.metadata.copy_(M0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ktimes = {}
    else:
        if not args.no_kernel_timing:
            # two event records per launch: every kernel costs these small steps some 30 us, Pass 1 alone a few
            mp.mpzch_set_kernel_timing(g.handle, 1 if args.all_kernel_timing else 3)
        t0 = time.perf_counter()
        for i in range(W, nb):
            one(i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ktimes = {} if args.no_kernel_timing else mp.mpzch_kernel_times(g.handle)
    K = len(batches) - W
    total = sum(b.numel() for _, b in batches[W:])
    cpu = None
    if args.cpu_steps > 0:
        import oracle
        o = oracle.Table(spec.num_slots, spec.max_probe, oracle.EVICT_TTL, spec.ttl, spec.hash_seed)
        for s, b in batches_np[:W]:
            o.remap(b, s)
        c0 = time.perf_counter()
        same = True
        for (s, b), og in list(zip(batches_np, outs))[W:]:
            r = o.remap(b, s)
            same = same and bool(np.array_equal(r.slots, og.cpu().numpy()))
        cpu = {"value": round(total / (time.perf_counter() - c0), 1), "unit": "ids/s", "cores": 1, "kind": "oracle",
               "sample": "all timed steps", "matches_gpu_out_slots": same}
    occ = int((g.identities >= 0).sum().item())
    roofline = None
    if "k_discover" in ktimes:
        distinct = float(sum(np.unique(b[b >= 0]).size for _, b in batches_np[W:]))
        alg, lines, hit_pos = training_alg_bytes(np, float(total), stats[W:].cpu().numpy().astype(np.float64), distinct,
                                                 mp.STAT_NAMES)
        ms_total, launches = ktimes["k_discover"]
        roofline = roofline_entry(args.workload, 1.0, "k_discover", ms_total / launches, alg / K, lines / K, hit_pos / K,
                                  note="the table lives in L2 / Infinity Cache and the step is bound by launches: the "
                                       "HBM fraction says little here")
    _emit("remapped IDs/sec (train insert+evict) at 1 GPU", total / elapsed, K, W, elapsed, name, ktimes, cpu,
          {"final_load": round(occ / spec.num_slots, 4)}, roofline)


def bench_jagged(args, np, torch, mp, wl, dev):
    """Config 5: 26 tables, one mpzch_remap_jagged call per step."""
    spec = wl.c5_spec(total_slots_cap=int(1_000_000_000 * args.scale), samples=max(int(65536 * args.scale), 64))
    K, W = min(args.steps, 5), min(args.warmup, 2)
    records = args.layout == "records"
    handles = [mp.mpzch_create_with_layout(t.num_slots, t.max_probe, (mp.EVICT_TTL, t.ttl), t.hash_seed,
                                           mp.LAYOUT_RECORDS if records else mp.LAYOUT_SEPARATE) for t in spec.tables]
    group = mp.mpzch_group_create(handles)
    if records:
        rec = [torch.empty(2 * t.num_slots, dtype=torch.int64, device=dev) for t in spec.tables]
        I, M = map(list, zip(*[mp.records_views(r, t.num_slots) for r, t in zip(rec, spec.tables)]))
    else:
        I = [torch.empty(t.num_slots, dtype=torch.int64, device=dev) for t in spec.tables]
        M = [torch.empty(t.num_slots, dtype=torch.int32, device=dev) for t in spec.tables]
    for h, i, m in zip(handles, I, M):
        mp.mpzch_init_tensors(h, i, m)
    T = len(spec.tables)
    data = [wl.c5_batch(spec, s) for s in range(1, W + K + 1)]
    dev_b = [(torch.from_numpy(v).to(dev), torch.from_numpy(o).to(dev), [int(x) for x in o]) for v, _, o in data]
    nmax = max(v.numel() for v, _, _ in dev_b)
    mp.mpzch_group_reserve(group, nmax)
    out = torch.empty(nmax, dtype=torch.int64, device=dev)
    ev = torch.empty(nmax, dtype=torch.int64, device=dev)
    nev = torch.zeros(T, dtype=torch.int64, device=dev)
    stats = torch.zeros((W + K, T * mp.STAT_COUNT), dtype=torch.int64, device=dev)

    # reset target of every table: bf16 rows of 16 values, one row per slot (32 GB for 1 B slots)
    emb = [torch.ones((t.num_slots, 16), dtype=torch.bfloat16, device=dev) for t in spec.tables]

    def one(i):
        v, o, eo = dev_b[i]
        mp.mpzch_remap_jagged(group, I, M, v, o, i + 1, out[: v.numel()], ev, eo, nev, stats[i])
        mp.mpzch_reset_rows_jagged(group, ev, eo, nev, emb)

    for i in range(W):
        one(i)
    torch.cuda.synchronize()
    mp.mpzch_group_set_kernel_timing(group, 1 if args.all_kernel_timing else 2)
    t0 = time.perf_counter()
    for i in range(W, W + K):
        one(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ktimes = mp.mpzch_group_kernel_times(group)
    total = sum(dev_b[i][0].numel() for i in range(W, W + K))
    st_all = stats[W:].cpu().numpy().reshape(K, T, mp.STAT_COUNT).astype(np.float64)
    st = st_all.sum(axis=(0, 1))
    roofline = None
    if "k_discover" in ktimes:
        alg = lines = stores = 0.0
        for f in range(T):                       # the byte accounting is per table: every table has its own probe lengths
            distinct = positions = 0.0
            for i in range(W, W + K):
                v, _, o = data[i]
                sl = v[int(o[f]):int(o[f + 1])]
                distinct += np.unique(sl[sl >= 0]).size
                positions += sl.size
            a, l, h = training_alg_bytes(np, positions, st_all[:, f, :], distinct, mp.STAT_NAMES)
            alg, lines, stores = alg + a, lines + l, stores + h
        ms_total, launches = ktimes["k_discover"]
        roofline = roofline_entry("c5" if records else "c5-separate", args.scale, "k_discover", ms_total / launches,
                                  alg / K, lines / K, stores / K, same_line=records,
                                  note="k_discover_tables; the small ones of the 26 tables live in L2 / Infinity Cache")
    _emit("remapped IDs/sec (train insert+evict) at 1 GPU", total / elapsed, K, W, elapsed,
          f"c5: 26 tables ({sum(t.num_slots for t in spec.tables)} slots in all), P=16, TTL=5, {spec.samples} samples, "
          f"pooling 1..50, about {total // K} values per step, one mpzch_remap_jagged + one mpzch_reset_rows_jagged call "
          f"per step (bf16 x16 rows per slot), identities+metadata as {'16-byte records' if records else 'two tensors'}",
          ktimes, None,
          {"totals_over_timed_steps": dict(zip(mp.STAT_NAMES, [int(x) for x in st]))}, roofline)


def bench_table1(args, np, torch, mp, wl, dev):
    """The collision-rate experiment of the paper's Table 1 as a workload: 150 M distinct ids are
    inserted (eviction off) into tables of 100 M .. 500 M slots at max_probe 8 .. 512; reports the
    collision rate of every cell next to the paper's and the insertion throughput against P."""
    n_ids = int(150_000_000 * args.scale)
    sizes_m = [100, 150, 200, 250, 300, 350, 400, 450, 500]
    probes = [8, 16, 32, 64, 128, 256, 512]
    golden = {}
    with open(os.path.join(ROOT, "tests", "golden", "table1_collision_rate.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                v = line.split()
                golden[int(v[0])] = dict(zip(probes, map(float, v[3:])))
    batch = max(int(262144 * args.scale), 1024)
    calls = (n_ids + batch - 1) // batch
    out = torch.empty(batch, dtype=torch.int64, device=dev)
    nev = torch.zeros(1, dtype=torch.int64, device=dev)
    stats = torch.zeros((calls, mp.STAT_COUNT), dtype=torch.int64, device=dev)
    ids_all = [wl.distinct_ids_device(lo, min(lo + batch, n_ids), dev) for lo in range(0, n_ids, batch)]
    rows, total_s, total_ids = [], 0.0, 0
    for sm in sizes_m:
        n_slots = int(sm * 1_000_000 * args.scale)
        I = torch.empty(n_slots, dtype=torch.int64, device=dev)
        M = torch.empty(n_slots, dtype=torch.int32, device=dev)
        for P in probes:
            h = mp.mpzch_create(n_slots, P, (mp.EVICT_NONE, 0), wl.HASH_SEED_BASE)
            mp.mpzch_reserve(h, batch)
            mp.mpzch_init_tensors(h, I, M)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k, ids in enumerate(ids_all):
                mp.mpzch_remap(h, I, M, ids, k, out[: ids.numel()], None, nev, stats[k])
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            coll = int(stats[:, mp.STAT_NAMES.index("collisions")].sum().item())
            rows.append({"table_millions": sm, "max_probe": P, "collision_pct": round(100.0 * coll / n_ids, 4),
                         "paper_pct": golden[sm][P], "ids_per_s": round(n_ids / dt, 1), "seconds": round(dt, 4)})
            log(f"[table1] {sm}M slots P={P}: {rows[-1]['collision_pct']:.4f}% (paper {golden[sm][P]:.4f}%) "
                f"{n_ids / dt / 1e9:.2f} G ids/s")
            total_s += dt
            total_ids += n_ids
            mp.mpzch_destroy(h)
        del I, M
    result = {
        "metric": "remapped IDs/sec (train insert, eviction off) at 1 GPU", "value": round(total_ids / total_s, 1),
        "unit": "ids/s", "n_gpus": 1, "steps": len(rows), "warmup": 0, "ms_per_step": round(total_s / len(rows) * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
        "config": {"workload": f"table1: {n_ids} distinct ids into 9 table sizes x 7 probe depths, {batch} ids per call, "
                               "eviction off", "scale": args.scale},
        "cells": rows, "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
