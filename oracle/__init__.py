"""ctypes front end of the MPZCH CPU oracle (TEST INFRASTRUCTURE, not the product).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library:
``mpzch_oracle.c`` is compiled with gcc and loaded here, state lives in numpy
arrays owned by the caller.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mpzch_oracle.c")
_LIB = os.path.join(_HERE, "libmpzch_oracle.so")

EVICT_NONE = 0
EVICT_TTL = 1
EVICT_LRU = 2
EVICT_TTL_EXPIRY = 3

STAT_NAMES = (
    "hit_pos", "miss_pos", "distinct_miss", "inserts",
    "evictions", "collisions", "invalid_pos", "hit_probe_sum", "miss_probe_sum",
)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (single thread, no tuning flags)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", tmp]
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("num_slots", ctypes.c_int64),
        ("max_probe", ctypes.c_int32),
        ("policy", ctypes.c_int32),
        ("ttl", ctypes.c_int32),
        ("pad_", ctypes.c_int32),
        ("hash_seed", ctypes.c_uint64),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p = ctypes.c_void_p
        lib.oracle_mix64.restype = ctypes.c_uint64
        lib.oracle_mix64.argtypes = [ctypes.c_uint64]
        lib.oracle_home.restype = ctypes.c_int64
        lib.oracle_home.argtypes = [ctypes.c_int64, ctypes.c_uint64, ctypes.c_int64]
        lib.oracle_remap.restype = ctypes.c_int
        lib.oracle_remap.argtypes = [ctypes.POINTER(_Cfg), p, p, p, ctypes.c_int64, ctypes.c_int32,
                                     p, p, ctypes.c_int64, p, p]
        lib.oracle_remap_ttls.restype = ctypes.c_int
        lib.oracle_remap_ttls.argtypes = [ctypes.POINTER(_Cfg), p, p, p, p, ctypes.c_int64, ctypes.c_int32,
                                          p, p, ctypes.c_int64, p, p]
        lib.oracle_lookup.restype = ctypes.c_int
        lib.oracle_lookup.argtypes = [ctypes.POINTER(_Cfg), p, p, ctypes.c_int64, p, p, p]
        lib.oracle_reset_rows.restype = ctypes.c_int
        lib.oracle_reset_rows.argtypes = [p, ctypes.c_int64, p, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int64, p]
        lib.oracle_check_state.restype = ctypes.c_int64
        lib.oracle_check_state.argtypes = [ctypes.POINTER(_Cfg), p, ctypes.c_int64, ctypes.c_int64, p, p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _i64(a) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype != np.int64 or not a.flags.c_contiguous:
        a = np.ascontiguousarray(a, dtype=np.int64)
    return a


def mix64(x: int) -> int:
    return int(_load().oracle_mix64(ctypes.c_uint64(x & 0xFFFFFFFFFFFFFFFF)))


def home(id_: int, seed: int, num_slots: int) -> int:
    return int(_load().oracle_home(ctypes.c_int64(id_), ctypes.c_uint64(seed), ctypes.c_int64(num_slots)))


@dataclass
class RemapResult:
    slots: np.ndarray          # int64[n]
    evicted: np.ndarray        # int64[num_evicted], claim order
    stats: dict


class Table:
    """One MPZCH table: config + caller-visible numpy state (identities, metadata)."""

    def __init__(self, num_slots: int, max_probe: int, policy: int = EVICT_TTL, ttl: int = 0,
                 hash_seed: int = 0, identities: np.ndarray | None = None,
                 metadata: np.ndarray | None = None):
        self.cfg = _Cfg(num_slots, max_probe, policy, ttl, 0, hash_seed & 0xFFFFFFFFFFFFFFFF)
        self.num_slots = num_slots
        self.max_probe = max_probe
        self.policy = policy
        self.ttl = ttl
        self.hash_seed = hash_seed
        # Sec. 3.1: identities start empty (-1); metadata start value is never consulted.
        self.identities = np.full(num_slots, -1, dtype=np.int64) if identities is None else identities
        self.metadata = np.full(num_slots, -1, dtype=np.int32) if metadata is None else metadata
        assert self.identities.dtype == np.int64 and self.identities.shape == (num_slots,)
        assert self.metadata.dtype == np.int32 and self.metadata.shape == (num_slots,)
        assert self.identities.flags.c_contiguous and self.metadata.flags.c_contiguous

    def remap(self, ids, step: int, ttls=None) -> RemapResult:
        """ttls: with EVICT_TTL_EXPIRY, int32 retention per position (per-feature TTL, Sec. 3.4)."""
        ids = _i64(ids)
        n = ids.shape[0]
        if ttls is not None:
            ttls = np.ascontiguousarray(ttls, dtype=np.int32)
            assert ttls.shape == (n,) and self.policy == EVICT_TTL_EXPIRY
        out = np.empty(n, dtype=np.int64)
        ev = np.empty(max(n, 1), dtype=np.int64)
        nev = np.zeros(1, dtype=np.int64)
        st = np.zeros(len(STAT_NAMES), dtype=np.int64)
        rc = _load().oracle_remap_ttls(ctypes.byref(self.cfg), _ptr(self.identities), _ptr(self.metadata),
                                       _ptr(ids), None if ttls is None else _ptr(ttls), n, step, _ptr(out),
                                       _ptr(ev), ev.shape[0], _ptr(nev), _ptr(st))
        if rc != 0:
            raise RuntimeError("oracle_remap failed")
        return RemapResult(out, ev[: int(nev[0])].copy(), dict(zip(STAT_NAMES, st.tolist())))

    def lookup(self, ids, want_stats: bool = False):
        """Returns (slots, found), or (slots, found, stats dict) with want_stats."""
        ids = _i64(ids)
        n = ids.shape[0]
        out = np.empty(n, dtype=np.int64)
        found = np.empty(n, dtype=np.uint8)
        st = np.zeros(len(STAT_NAMES), dtype=np.int64)
        rc = _load().oracle_lookup(ctypes.byref(self.cfg), _ptr(self.identities), _ptr(ids), n,
                                   _ptr(out), _ptr(found), _ptr(st))
        if rc != 0:
            raise RuntimeError("oracle_lookup failed")
        if want_stats:
            return out, found, dict(zip(STAT_NAMES, st.tolist()))
        return out, found

    def check_state(self, lo: int = 0, hi: int | None = None):
        """Returns (violations, occupied, first_bad_slot) over slots [lo, hi)."""
        hi = self.num_slots if hi is None else hi
        occ = np.zeros(1, dtype=np.int64)
        fb = np.zeros(1, dtype=np.int64)
        bad = _load().oracle_check_state(ctypes.byref(self.cfg), _ptr(self.identities), lo, hi,
                                         _ptr(occ), _ptr(fb))
        return int(bad), int(occ[0]), int(fb[0])


def remap_jagged(tables, values, feature_offsets, step: int, ttls=None):
    """Keyed-jagged batch: feature f owns values[offsets[f]:offsets[f+1]] and table f.

    Tables are independent (Sec. 3.6: operations stay local to a table's shard),
    so the batch is the per-table remap applied to each slice.
    ttls: optional per-value retention (Sec. 3.4, per-feature TTL) for the expiry-step tables.
    Returns (slots int64[total], [evicted arrays per table], [stats per table]).
    """
    values = _i64(values)
    offs = np.asarray(feature_offsets, dtype=np.int64)
    out = np.empty(values.shape[0], dtype=np.int64)
    evs, sts = [], []
    for f, t in enumerate(tables):
        lo, hi = int(offs[f]), int(offs[f + 1])
        # per-value retention applies to tables that store expiry steps; the others have their own ttl
        use = ttls is not None and t.policy == EVICT_TTL_EXPIRY
        r = t.remap(values[lo:hi], step, np.asarray(ttls)[lo:hi] if use else None)
        out[lo:hi] = r.slots
        evs.append(r.evicted)
        sts.append(r.stats)
    return out, evs, sts


def reset_rows(slots, rows: np.ndarray, init_row: np.ndarray | None = None):
    """rows: 2-D C-contiguous array; rows[slot % num_rows, :] <- init_row (zeros if None)."""
    slots = _i64(slots)
    assert rows.ndim == 2 and rows.flags.c_contiguous
    num_rows = rows.shape[0]
    row_bytes = rows.shape[1] * rows.itemsize
    init_p = None
    if init_row is not None:
        init_row = np.ascontiguousarray(init_row, dtype=rows.dtype)
        assert init_row.nbytes == row_bytes
        init_p = _ptr(init_row)
    rc = _load().oracle_reset_rows(_ptr(slots), slots.shape[0], _ptr(rows), num_rows, row_bytes,
                                   row_bytes, init_p)
    if rc != 0:
        raise RuntimeError("oracle_reset_rows failed")


def collect_delta(table: Table, since_step: int):
    """Sec. 3.8 sparse delta: (slots, ids) of every occupied slot seen at or after since_step, ascending slot."""
    slots = np.nonzero((table.identities >= 0) & (table.metadata >= since_step))[0].astype(np.int64)
    return slots, table.identities[slots].copy()


def gather_rows(slots, rows: np.ndarray) -> np.ndarray:
    return rows[_i64(slots) % rows.shape[0]].copy()


def apply_delta(identities: np.ndarray, slots, ids, rows: np.ndarray | None = None, delta_rows=None):
    """Sec. 3.8: identities entries are updated together with the embedding rows they belong to."""
    slots = _i64(slots)
    if rows is not None:
        rows[slots % rows.shape[0]] = delta_rows
    identities[slots] = _i64(ids)
