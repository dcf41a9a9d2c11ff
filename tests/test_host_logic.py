"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_17050_amd", "libmpzch.so")
HEADER = os.path.join(ROOT, "include", "mpzch.h")


@pytest.fixture(scope="module")
def binding():
    if not os.path.exists(LIB):
        from paper_2602_17050_amd import build
        build.build_library()
    from paper_2602_17050_amd import binding as b
    b.load_library()
    return b


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mpzch_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(binding):
    lib = ctypes.CDLL(LIB)
    names = declared_symbols()
    assert "mpzch_create" in names and "mpzch_remap" in names and "mpzch_lookup" in names
    assert "mpzch_reset_rows" in names and "mpzch_remap_jagged" in names
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTED) == set(names)


def test_binding_uses_the_c_abi_names(binding):
    for n in binding.EXPORTED:
        assert callable(getattr(binding, n)), n


def test_create_validates_arguments_without_a_gpu(binding):
    b = binding
    h = b.mpzch_create(4096, 8, (b.EVICT_TTL, 3), 0x5EED)
    b.mpzch_destroy(h)
    h = b.mpzch_create(10, 64, (b.EVICT_NONE, 0), 1)        # max_probe > num_slots is accepted
    b.mpzch_destroy(h)
    for args in [(0, 8, (b.EVICT_TTL, 3)), (16, 0, (b.EVICT_TTL, 3)), (16, 8, (b.EVICT_TTL, -1)),
                 (16, 8, (7, 0)), (16, (1 << 20) + 1, (b.EVICT_NONE, 0))]:
        with pytest.raises(b.MpzchError) as e:
            b.mpzch_create(args[0], args[1], args[2], 0)
        assert e.value.status == 1
    b.mpzch_destroy(b.mpzch_create(16, 8, (b.EVICT_LRU, 0), 0))
    with pytest.raises(b.MpzchError) as e:
        b.mpzch_create(5000, 1025, (b.EVICT_LRU, 0), 0)      # LRU: max_probe <= 1024
    assert e.value.status == 4
    assert b.mpzch_status_string(0) == "ok"
    assert b.mpzch_status_string(1) == "invalid argument"


def test_entry_points_reject_bad_arguments_before_touching_the_gpu(binding):
    """Checks that run before the first HIP call: NULL handles and required pointers, sizes out of range, a slot
    count beyond MPZCH_MAX_SLOTS, a table that would reach past the 48 bits the kernels keep of an address."""
    b = binding
    lib = b.load_library()
    vp = ctypes.c_void_p
    h = b.mpzch_create(1000, 8, (b.EVICT_TTL, 1), 0)
    fake = vp(0x10000)                                        # never dereferenced: every call below fails first
    INVALID = 1
    assert lib.mpzch_remap(None, fake, fake, fake, 4, 1, fake, fake, 4, fake, None, None) == INVALID
    assert lib.mpzch_remap(h, None, fake, fake, 4, 1, fake, fake, 4, fake, None, None) == INVALID
    assert lib.mpzch_remap(h, fake, fake, fake, -1, 1, fake, fake, 4, fake, None, None) == INVALID
    assert lib.mpzch_remap(h, fake, fake, fake, (1 << 30) + 1, 1, fake, fake, 4, fake, None, None) == INVALID
    assert lib.mpzch_remap(h, fake, fake, fake, 4, -1, fake, fake, 4, fake, None, None) == INVALID      # step < 0
    assert lib.mpzch_remap(h, fake, fake, fake, 4, 1, None, fake, 4, fake, None, None) == INVALID       # no out_slots
    assert lib.mpzch_remap(h, fake, fake, fake, 4, 1, fake, None, 4, fake, None, None) == INVALID       # list of 4, no pointer
    high = vp((1 << 48) - 4096)                                # identities would end beyond 2^48
    assert lib.mpzch_remap(h, high, fake, fake, 4, 1, fake, fake, 4, fake, None, None) == INVALID
    assert lib.mpzch_lookup(h, high, fake, 4, fake, None, None) == INVALID
    assert lib.mpzch_remap_reset(h, fake, fake, fake, 4, 1, fake, fake, 4, fake, None, None, 10, 16, 16, None, None) == INVALID
    assert lib.mpzch_remap_reset(h, fake, fake, fake, 4, 1, fake, fake, 4, fake, None, fake, 0, 16, 16, None, None) == INVALID
    assert lib.mpzch_remap_reset(h, fake, fake, fake, 4, 1, fake, fake, 4, fake, None, fake, 10, 6, 8, None, None) == INVALID
    assert lib.mpzch_remap_noalloc(h, fake, fake, fake, b.NOALLOC_MAX_BATCH + 1, 1, fake, fake, 4, fake, None, None) == 5
    assert lib.mpzch_lookup(None, fake, fake, 4, fake, None, None) == INVALID
    assert lib.mpzch_lookup_gather(h, fake, fake, 4, None, 10, 16, 16, fake, None, None, None) == INVALID  # no rows
    assert lib.mpzch_reset_rows(fake, fake, 4, fake, 10, 6, 8, None, None) == INVALID                       # 6-byte rows
    assert lib.mpzch_reserve(h, -1) == INVALID
    b.mpzch_destroy(h)
    with pytest.raises(b.MpzchError) as e:
        b.mpzch_create((1 << 40) + 1, 8, (b.EVICT_TTL, 1), 0)
    assert e.value.status == INVALID
    hr = b.mpzch_create_with_layout(1000, 8, (b.EVICT_TTL, 1), 0, b.LAYOUT_RECORDS)
    assert lib.mpzch_lookup(hr, vp(0x10008), fake, 4, fake, None, None) == INVALID      # records not 16-byte aligned
    assert lib.mpzch_remap(hr, vp(0x10000), vp(0x10004), fake, 4, 1, fake, fake, 4, fake, None, None) == INVALID  # metadata elsewhere
    b.mpzch_destroy(hr)
    with pytest.raises(b.MpzchError):
        b.mpzch_create_with_layout(1000, 8, (b.EVICT_TTL, 1), 0, 2)


def test_group_create_validates_arguments(binding):
    b = binding
    hs = [b.mpzch_create(100 + i, 4, (b.EVICT_TTL, 1), i) for i in range(3)]
    g = b.mpzch_group_create(hs)
    for h in hs:
        b.mpzch_destroy(h)                                   # the group keeps its own copy of the configs
    b.mpzch_group_destroy(g)
    with pytest.raises(b.MpzchError):
        b.mpzch_group_create([])
    h = b.mpzch_create(100, 4, (b.EVICT_LRU, 0), 0)
    b.mpzch_group_destroy(b.mpzch_group_create([h]))          # every policy may sit in a group
    b.mpzch_destroy(h)


def test_missing_library_fails_loudly(binding, tmp_path):
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "libmpzch.so"))
