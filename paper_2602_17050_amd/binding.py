"""Thin ctypes binding over libmpzch.so (the C ABI of include/mpzch.h).

Argument marshalling only: torch tensors supply device memory and the current
stream; every step of the path runs in the library's HIP kernels.  There is no
fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmpzch.so")

EVICT_NONE, EVICT_TTL, EVICT_LRU, EVICT_TTL_EXPIRY = 0, 1, 2, 3
STAT_NAMES = ("hit_pos", "miss_pos", "distinct_miss", "inserts",
              "evictions", "collisions", "invalid_pos", "hit_probe_sum", "miss_probe_sum")
STAT_COUNT = len(STAT_NAMES)

EXPORTED = (
    "mpzch_create", "mpzch_destroy", "mpzch_reserve", "mpzch_init_tensors", "mpzch_remap",
    "mpzch_lookup", "mpzch_reset_rows", "mpzch_group_create", "mpzch_group_destroy",
    "mpzch_group_reserve", "mpzch_remap_jagged", "mpzch_set_kernel_timing", "mpzch_kernel_times",
    "mpzch_group_set_kernel_timing", "mpzch_group_kernel_times", "mpzch_status_string",
    "mpzch_remap_feature_ttl", "mpzch_reset_rows_multi", "mpzch_lookup_gather", "mpzch_collect_delta", "mpzch_gather_rows", "mpzch_apply_delta",
    "mpzch_remap_jagged_feature_ttl", "mpzch_lookup_jagged", "mpzch_reset_rows_jagged",
    "mpzch_remap_noalloc", "mpzch_lookup_stats", "mpzch_create_with_layout", "mpzch_remap_reset",
)
LAYOUT_SEPARATE, LAYOUT_RECORDS = 0, 1
NOALLOC_MAX_BATCH = 262144


class MpzchError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {mpzch_status_string(status)} ({status})")


class _Policy(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("ttl", ctypes.c_int32)]


class _Rows(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_void_p), ("num_rows", ctypes.c_int64), ("row_bytes", ctypes.c_int64),
                ("row_stride_bytes", ctypes.c_int64), ("init_row", ctypes.c_void_p)]


_lib = None


def load_library(path: str | None = None):
    """Loads the in-tree HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("MPZCH_LIBRARY") or _LIB_PATH   # env override: another build of the same ABI
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2602_17050_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    lib.mpzch_create.argtypes = [i64, i32, _Policy, ctypes.c_uint64, ctypes.POINTER(vp)]
    lib.mpzch_create_with_layout.argtypes = [i64, i32, _Policy, ctypes.c_uint64, i32, ctypes.POINTER(vp)]
    lib.mpzch_destroy.argtypes = [vp]
    lib.mpzch_reserve.argtypes = [vp, i64]
    lib.mpzch_init_tensors.argtypes = [vp, vp, vp, vp]
    lib.mpzch_remap.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp, i64, vp, vp, vp]
    lib.mpzch_remap_noalloc.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp, i64, vp, vp, vp]
    lib.mpzch_remap_reset.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp, i64, vp, vp, vp, i64, i64, i64, vp, vp]
    lib.mpzch_remap_feature_ttl.argtypes = [vp, vp, vp, vp, vp, i64, i32, vp, vp, i64, vp, vp, vp]
    lib.mpzch_lookup.argtypes = [vp, vp, vp, i64, vp, vp, vp]
    lib.mpzch_lookup_stats.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp]
    lib.mpzch_reset_rows.argtypes = [vp, vp, i64, vp, i64, i64, i64, vp, vp]
    lib.mpzch_reset_rows_multi.argtypes = [vp, vp, i64, ctypes.POINTER(_Rows), i32, vp]
    lib.mpzch_lookup_gather.argtypes = [vp, vp, vp, i64, vp, i64, i64, i64, vp, vp, vp, vp]
    lib.mpzch_collect_delta.argtypes = [vp, vp, vp, i32, vp, vp, i64, vp, vp]
    lib.mpzch_gather_rows.argtypes = [vp, vp, i64, vp, i64, i64, i64, vp, vp]
    lib.mpzch_apply_delta.argtypes = [vp, i64, vp, vp, vp, i64, vp, i64, i64, i64, vp, vp]
    lib.mpzch_group_create.argtypes = [ctypes.POINTER(vp), i32, ctypes.POINTER(vp)]
    lib.mpzch_group_destroy.argtypes = [vp]
    lib.mpzch_group_reserve.argtypes = [vp, i64]
    lib.mpzch_remap_jagged.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp, i64, i32, vp, vp,
                                       ctypes.POINTER(i64), vp, vp, vp]
    lib.mpzch_remap_jagged_feature_ttl.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp, vp, i64, i32, vp,
                                                   vp, ctypes.POINTER(i64), vp, vp, vp]
    lib.mpzch_reset_rows_jagged.argtypes = [vp, vp, ctypes.POINTER(i64), vp, ctypes.POINTER(_Rows), vp]
    lib.mpzch_lookup_jagged.argtypes = [vp, ctypes.POINTER(vp), vp, vp, i64, vp, vp, vp]
    for name in ("mpzch_kernel_times", "mpzch_group_kernel_times"):
        getattr(lib, name).argtypes = [vp, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(i64), i32, ctypes.POINTER(i32)]
    lib.mpzch_set_kernel_timing.argtypes = [vp, i32]
    lib.mpzch_group_set_kernel_timing.argtypes = [vp, i32]
    lib.mpzch_status_string.argtypes = [i32]
    lib.mpzch_status_string.restype = ctypes.c_char_p
    for name in EXPORTED:
        if name != "mpzch_status_string":
            getattr(lib, name).restype = ctypes.c_int32
    if path == _LIB_PATH:
        _lib = lib
    return lib


def mpzch_status_string(status: int) -> str:
    return load_library().mpzch_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise MpzchError(status, what)


def _ptr(t, dtype=None):
    if t is None:
        return None
    # dense tensors, or the strided views of a table kept as 16-byte records (identities: every second
    # int64, metadata: every fourth int32)
    assert t.is_cuda and (t.is_contiguous() or (t.dim() == 1 and t.stride(0) in (2, 4))), "device, dense tensors only"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


# ----------------------------------------------------------------------------- C-ABI names
def mpzch_create(num_slots: int, max_probe: int, eviction_policy=(EVICT_TTL, 0), hash_seed: int = 0):
    """Returns an opaque handle (ctypes.c_void_p).  eviction_policy = (kind, ttl)."""
    h = ctypes.c_void_p()
    pol = _Policy(int(eviction_policy[0]), int(eviction_policy[1]))
    _check(load_library().mpzch_create(num_slots, max_probe, pol, ctypes.c_uint64(hash_seed & (2 ** 64 - 1)),
                                       ctypes.byref(h)), "mpzch_create")
    return h


def mpzch_create_with_layout(num_slots: int, max_probe: int, eviction_policy=(EVICT_TTL, 0), hash_seed: int = 0,
                             layout: int = LAYOUT_SEPARATE):
    h = ctypes.c_void_p()
    pol = _Policy(int(eviction_policy[0]), int(eviction_policy[1]))
    _check(load_library().mpzch_create_with_layout(num_slots, max_probe, pol, ctypes.c_uint64(hash_seed & (2 ** 64 - 1)),
                                                   int(layout), ctypes.byref(h)), "mpzch_create_with_layout")
    return h


def records_views(records, num_slots: int):
    """(identities, metadata) views of a table kept as num_slots 16-byte records in an int64[2 * num_slots] tensor."""
    return records.view(num_slots, 2)[:, 0], records.view(torch.int32).view(num_slots, 4)[:, 2]


def mpzch_destroy(handle):
    _check(load_library().mpzch_destroy(handle), "mpzch_destroy")


def mpzch_reserve(handle, max_n: int):
    _check(load_library().mpzch_reserve(handle, max_n), "mpzch_reserve")


def mpzch_init_tensors(handle, identities, metadata=None):
    _check(load_library().mpzch_init_tensors(handle, _ptr(identities, torch.int64), _ptr(metadata, torch.int32),
                                             _stream()), "mpzch_init_tensors")


def mpzch_remap(handle, identities, metadata, ids, step: int, out_slots, out_evicted_slots, out_num_evicted,
                out_stats=None):
    n = ids.numel()
    cap = 0 if out_evicted_slots is None else out_evicted_slots.numel()
    _check(load_library().mpzch_remap(handle, _ptr(identities, torch.int64), _ptr(metadata, torch.int32),
                                      _ptr(ids, torch.int64), n, step, _ptr(out_slots, torch.int64),
                                      _ptr(out_evicted_slots, torch.int64), cap, _ptr(out_num_evicted, torch.int64),
                                      _ptr(out_stats, torch.int64), _stream()), "mpzch_remap")


def mpzch_remap_reset(handle, identities, metadata, ids, step: int, out_slots, out_evicted_slots, out_num_evicted,
                      out_stats, rows, init_row=None, num_rows: int | None = None):
    """mpzch_remap that also resets rows[slot mod num_rows] of every slot it evicts; rows: 2-D tensor (num_rows, dim)."""
    n = ids.numel()
    cap = 0 if out_evicted_slots is None else out_evicted_slots.numel()
    assert rows.dim() == 2 and rows.stride(1) == 1 and rows.is_cuda
    nrows = rows.shape[0] if num_rows is None else num_rows
    row_bytes = rows.shape[1] * rows.element_size()
    stride = rows.stride(0) * rows.element_size()
    if init_row is not None:
        assert init_row.is_cuda and init_row.is_contiguous() and init_row.numel() * init_row.element_size() == row_bytes
    _check(load_library().mpzch_remap_reset(handle, _ptr(identities, torch.int64), _ptr(metadata, torch.int32),
                                            _ptr(ids, torch.int64), n, step, _ptr(out_slots, torch.int64),
                                            _ptr(out_evicted_slots, torch.int64), cap, _ptr(out_num_evicted, torch.int64),
                                            _ptr(out_stats, torch.int64), ctypes.c_void_p(rows.data_ptr()), nrows,
                                            row_bytes, stride,
                                            None if init_row is None else ctypes.c_void_p(init_row.data_ptr()),
                                            _stream()), "mpzch_remap_reset")


def mpzch_remap_noalloc(handle, identities, metadata, ids, step: int, out_slots, out_evicted_slots, out_num_evicted,
                        out_stats=None):
    n = ids.numel()
    cap = 0 if out_evicted_slots is None else out_evicted_slots.numel()
    _check(load_library().mpzch_remap_noalloc(handle, _ptr(identities, torch.int64), _ptr(metadata, torch.int32),
                                              _ptr(ids, torch.int64), n, step, _ptr(out_slots, torch.int64),
                                              _ptr(out_evicted_slots, torch.int64), cap,
                                              _ptr(out_num_evicted, torch.int64), _ptr(out_stats, torch.int64),
                                              _stream()), "mpzch_remap_noalloc")


def mpzch_remap_feature_ttl(handle, identities, metadata, ids, ttls, step: int, out_slots, out_evicted_slots,
                            out_num_evicted, out_stats=None):
    n = ids.numel()
    cap = 0 if out_evicted_slots is None else out_evicted_slots.numel()
    assert ttls is None or ttls.numel() == n
    _check(load_library().mpzch_remap_feature_ttl(handle, _ptr(identities, torch.int64), _ptr(metadata, torch.int32),
                                                  _ptr(ids, torch.int64), _ptr(ttls, torch.int32), n, step,
                                                  _ptr(out_slots, torch.int64), _ptr(out_evicted_slots, torch.int64),
                                                  cap, _ptr(out_num_evicted, torch.int64),
                                                  _ptr(out_stats, torch.int64), _stream()), "mpzch_remap_feature_ttl")


def mpzch_lookup(handle, identities, ids, out_slots, out_found=None):
    _check(load_library().mpzch_lookup(handle, _ptr(identities, torch.int64), _ptr(ids, torch.int64), ids.numel(),
                                       _ptr(out_slots, torch.int64), _ptr(out_found, torch.uint8), _stream()),
           "mpzch_lookup")


def mpzch_lookup_stats(handle, identities, ids, out_slots, out_found, out_stats):
    _check(load_library().mpzch_lookup_stats(handle, _ptr(identities, torch.int64), _ptr(ids, torch.int64), ids.numel(),
                                             _ptr(out_slots, torch.int64), _ptr(out_found, torch.uint8),
                                             _ptr(out_stats, torch.int64), _stream()), "mpzch_lookup_stats")


def mpzch_reset_rows(slots, num_slots_dev, rows, init_row=None, num_rows: int | None = None):
    """rows: 2-D tensor (num_rows, dim); row = slot mod num_rows."""
    assert rows.dim() == 2 and rows.stride(1) == 1
    nrows = rows.shape[0] if num_rows is None else num_rows
    row_bytes = rows.shape[1] * rows.element_size()
    stride = rows.stride(0) * rows.element_size()
    if init_row is not None:
        assert init_row.is_cuda and init_row.is_contiguous() and init_row.numel() * init_row.element_size() == row_bytes
    _check(load_library().mpzch_reset_rows(_ptr(slots, torch.int64), _ptr(num_slots_dev, torch.int64), slots.numel(),
                                           ctypes.c_void_p(rows.data_ptr()), nrows, row_bytes, stride,
                                           None if init_row is None else ctypes.c_void_p(init_row.data_ptr()),
                                           _stream()), "mpzch_reset_rows")


def _row_geometry(rows):
    assert rows.dim() == 2 and rows.stride(1) == 1 and rows.is_cuda
    return rows.shape[0], rows.shape[1] * rows.element_size(), rows.stride(0) * rows.element_size()


def mpzch_reset_rows_multi(slots, num_slots_dev, tensors, init_rows=None):
    """tensors: list of 2-D device tensors (weights, optimizer state, ...), reset in one launch."""
    init_rows = init_rows or [None] * len(tensors)
    arr = (_Rows * len(tensors))()
    for k, (t, init) in enumerate(zip(tensors, init_rows)):
        n, rb, st = _row_geometry(t)
        arr[k] = _Rows(t.data_ptr(), n, rb, st, None if init is None else init.data_ptr())
    _check(load_library().mpzch_reset_rows_multi(_ptr(slots, torch.int64), _ptr(num_slots_dev, torch.int64),
                                                 slots.numel(), arr, len(tensors), _stream()), "mpzch_reset_rows_multi")


def mpzch_lookup_gather(handle, identities, ids, rows, out_rows, out_slots=None, out_found=None):
    n, rb, st = _row_geometry(rows)
    assert out_rows.is_contiguous() and out_rows.numel() * out_rows.element_size() == ids.numel() * rb
    _check(load_library().mpzch_lookup_gather(handle, _ptr(identities, torch.int64), _ptr(ids, torch.int64), ids.numel(),
                                              ctypes.c_void_p(rows.data_ptr()), n, rb, st,
                                              ctypes.c_void_p(out_rows.data_ptr()), _ptr(out_slots, torch.int64),
                                              _ptr(out_found, torch.uint8), _stream()), "mpzch_lookup_gather")


def mpzch_collect_delta(handle, identities, metadata, since_step: int, out_slots, out_ids, out_count):
    _check(load_library().mpzch_collect_delta(handle, _ptr(identities, torch.int64), _ptr(metadata, torch.int32),
                                              since_step, _ptr(out_slots, torch.int64), _ptr(out_ids, torch.int64),
                                              out_slots.numel(), _ptr(out_count, torch.int64), _stream()),
           "mpzch_collect_delta")


def mpzch_gather_rows(slots, count_dev, rows, out_rows):
    n, rb, st = _row_geometry(rows)
    assert out_rows.is_contiguous()
    _check(load_library().mpzch_gather_rows(_ptr(slots, torch.int64), _ptr(count_dev, torch.int64), slots.numel(),
                                            ctypes.c_void_p(rows.data_ptr()), n, rb, st,
                                            ctypes.c_void_p(out_rows.data_ptr()), _stream()), "mpzch_gather_rows")


def mpzch_apply_delta(identities, slots, ids, count_dev, rows=None, delta_rows=None):
    if rows is not None:
        n, rb, st = _row_geometry(rows)
        rp, dp = ctypes.c_void_p(rows.data_ptr()), ctypes.c_void_p(delta_rows.data_ptr())
    else:
        n, rb, st, rp, dp = 0, 0, 0, None, None
    _check(load_library().mpzch_apply_delta(_ptr(identities, torch.int64), identities.numel(), _ptr(slots, torch.int64),
                                            _ptr(ids, torch.int64), _ptr(count_dev, torch.int64), slots.numel(),
                                            rp, n, rb, st, dp, _stream()), "mpzch_apply_delta")


def mpzch_group_create(handles):
    arr = (ctypes.c_void_p * len(handles))(*[h.value for h in handles])
    g = ctypes.c_void_p()
    _check(load_library().mpzch_group_create(arr, len(handles), ctypes.byref(g)), "mpzch_group_create")
    return g


def mpzch_group_destroy(group):
    _check(load_library().mpzch_group_destroy(group), "mpzch_group_destroy")


def mpzch_group_reserve(group, max_total_values: int):
    _check(load_library().mpzch_group_reserve(group, max_total_values), "mpzch_group_reserve")


def mpzch_remap_jagged_feature_ttl(group, identities, metadata, values, ttls, feature_offsets, step: int, out_slots,
                                   out_evicted_slots, evicted_offsets, out_num_evicted, out_stats=None):
    """identities / metadata: lists of device tensors; ttls: int32 per value or None;
    evicted_offsets: host list of ints."""
    T = len(identities)
    ip = (ctypes.c_void_p * T)(*[t.data_ptr() for t in identities])
    mp = (ctypes.c_void_p * T)(*[t.data_ptr() for t in metadata])
    eo = (ctypes.c_int64 * (T + 1))(*[int(x) for x in evicted_offsets])
    _check(load_library().mpzch_remap_jagged_feature_ttl(
        group, ip, mp, _ptr(values, torch.int64), _ptr(ttls, torch.int32), _ptr(feature_offsets, torch.int64),
        values.numel(), step, _ptr(out_slots, torch.int64), _ptr(out_evicted_slots, torch.int64), eo,
        _ptr(out_num_evicted, torch.int64), _ptr(out_stats, torch.int64), _stream()), "mpzch_remap_jagged_feature_ttl")


def mpzch_remap_jagged(group, identities, metadata, values, feature_offsets, step: int, out_slots,
                       out_evicted_slots, evicted_offsets, out_num_evicted, out_stats=None):
    """identities / metadata: lists of device tensors; evicted_offsets: host list of ints."""
    T = len(identities)
    ip = (ctypes.c_void_p * T)(*[t.data_ptr() for t in identities])
    mp = (ctypes.c_void_p * T)(*[t.data_ptr() for t in metadata])
    eo = (ctypes.c_int64 * (T + 1))(*[int(x) for x in evicted_offsets])
    _check(load_library().mpzch_remap_jagged(group, ip, mp, _ptr(values, torch.int64),
                                             _ptr(feature_offsets, torch.int64), values.numel(), step,
                                             _ptr(out_slots, torch.int64), _ptr(out_evicted_slots, torch.int64), eo,
                                             _ptr(out_num_evicted, torch.int64), _ptr(out_stats, torch.int64),
                                             _stream()), "mpzch_remap_jagged")


def mpzch_reset_rows_jagged(group, evicted_slots, evicted_offsets, num_evicted, tensors, init_rows=None):
    """tensors: one 2-D device tensor (or None) per table of the group; evicted_offsets: host list of ints."""
    T = len(tensors)
    init_rows = init_rows or [None] * T
    arr = (_Rows * T)()
    for k, (t, init) in enumerate(zip(tensors, init_rows)):
        if t is None:
            arr[k] = _Rows(None, 0, 0, 0, None)
        else:
            n, rb, st = _row_geometry(t)
            arr[k] = _Rows(t.data_ptr(), n, rb, st, None if init is None else init.data_ptr())
    eo = (ctypes.c_int64 * (T + 1))(*[int(x) for x in evicted_offsets])
    _check(load_library().mpzch_reset_rows_jagged(group, _ptr(evicted_slots, torch.int64), eo,
                                                  _ptr(num_evicted, torch.int64), arr, _stream()),
           "mpzch_reset_rows_jagged")


def mpzch_lookup_jagged(group, identities, values, feature_offsets, out_slots, out_found=None):
    """identities: list of device tensors, one per table of the group."""
    T = len(identities)
    ip = (ctypes.c_void_p * T)(*[t.data_ptr() for t in identities])
    _check(load_library().mpzch_lookup_jagged(group, ip, _ptr(values, torch.int64), _ptr(feature_offsets, torch.int64),
                                              values.numel(), _ptr(out_slots, torch.int64), _ptr(out_found, torch.uint8),
                                              _stream()), "mpzch_lookup_jagged")


def _times(fn, handle):
    cap = 16
    names = (ctypes.c_char_p * cap)()
    ms = (ctypes.c_double * cap)()
    cnt = (ctypes.c_int64 * cap)()
    k = ctypes.c_int32()
    _check(fn(handle, names, ms, cnt, cap, ctypes.byref(k)), "kernel_times")
    return {names[i].decode(): (ms[i], cnt[i]) for i in range(k.value)}


def mpzch_set_kernel_timing(handle, enable):
    """enable: 0 / False = off, 1 / True = every kernel, 2 = the Pass-1 kernel only, 3 = the Pass-1 kernel of every fourth call."""
    _check(load_library().mpzch_set_kernel_timing(handle, int(enable)), "mpzch_set_kernel_timing")


def mpzch_kernel_times(handle):
    """{kernel name: (total ms, launches)} since the last read-out; synchronises."""
    return _times(load_library().mpzch_kernel_times, handle)


def mpzch_group_set_kernel_timing(group, enable):
    _check(load_library().mpzch_group_set_kernel_timing(group, int(enable)), "mpzch_group_set_kernel_timing")


def mpzch_group_kernel_times(group):
    return _times(load_library().mpzch_group_kernel_times, group)


# ----------------------------------------------------------------------------- convenience
class MpzchTable:
    """Owns the tensors of one table (torch device memory) and its handle."""

    def __init__(self, num_slots, max_probe, kind=EVICT_TTL, ttl=0, hash_seed=0, device="cuda", max_batch=0,
                 layout=LAYOUT_SEPARATE):
        self.num_slots, self.max_probe, self.kind, self.ttl, self.hash_seed = num_slots, max_probe, kind, ttl, hash_seed
        self.layout = layout
        self.handle = mpzch_create_with_layout(num_slots, max_probe, (kind, ttl), hash_seed, layout)
        if layout == LAYOUT_RECORDS:
            self.records = torch.empty(2 * num_slots, dtype=torch.int64, device=device)
            self.identities, self.metadata = records_views(self.records, num_slots)
        else:
            self.identities = torch.empty(num_slots, dtype=torch.int64, device=device)
            self.metadata = torch.empty(num_slots, dtype=torch.int32, device=device)
        mpzch_init_tensors(self.handle, self.identities, self.metadata)
        self.num_evicted = torch.zeros(1, dtype=torch.int64, device=device)
        self.stats = torch.zeros(STAT_COUNT, dtype=torch.int64, device=device)
        self._evicted = None
        if max_batch:
            mpzch_reserve(self.handle, max_batch)
            self._evicted = torch.empty(max_batch, dtype=torch.int64, device=device)

    def remap(self, ids, step, out_slots=None, ttls=None):
        n = ids.numel()
        if out_slots is None:
            out_slots = torch.empty(n, dtype=torch.int64, device=ids.device)
        if self._evicted is None or self._evicted.numel() < n:
            self._evicted = torch.empty(max(n, 1), dtype=torch.int64, device=ids.device)
        mpzch_remap_feature_ttl(self.handle, self.identities, self.metadata, ids, ttls, step, out_slots,
                                self._evicted, self.num_evicted, self.stats)
        return out_slots

    def remap_reset(self, ids, step, rows, init_row=None, out_slots=None):
        """remap + reset of the evicted slots' rows in one call (mpzch_remap_reset)"""
        n = ids.numel()
        if out_slots is None:
            out_slots = torch.empty(n, dtype=torch.int64, device=ids.device)
        if self._evicted is None or self._evicted.numel() < n:
            self._evicted = torch.empty(max(n, 1), dtype=torch.int64, device=ids.device)
        mpzch_remap_reset(self.handle, self.identities, self.metadata, ids, step, out_slots, self._evicted,
                          self.num_evicted, self.stats, rows, init_row)
        return out_slots

    @property
    def evicted(self):
        """Evicted slots of the last remap (synchronises to read the count)."""
        return self._evicted[: int(self.num_evicted.item())]

    def reset_rows(self, rows, init_row=None):
        mpzch_reset_rows(self._evicted, self.num_evicted, rows, init_row)

    def lookup(self, ids, want_found=True):
        out = torch.empty(ids.numel(), dtype=torch.int64, device=ids.device)
        found = torch.empty(ids.numel(), dtype=torch.uint8, device=ids.device) if want_found else None
        mpzch_lookup(self.handle, self.identities, ids, out, found)
        return out, found

    def stats_dict(self):
        return dict(zip(STAT_NAMES, self.stats.tolist()))

    def close(self):
        if self.handle is not None:
            mpzch_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
