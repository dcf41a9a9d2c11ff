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
