"""The C-ABI library loads, exports every symbol the header declares, and its host-side checks that
need no device behave.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2601_11553_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2601_11553_amd.build import build_library
        build_library()
    return binding.load_library()


def test_header_symbols_are_exported(lib):
    from paper_2601_11553_amd import binding
    text = open(os.path.join(ROOT, "include", "percache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(percache_[a-z0-9_]+)\s*\(", text)))
    assert len(declared) >= 16
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in percache.h but not exported"
    assert sorted(binding.EXPORTS) == declared


def test_arena_bytes_and_config_validation(lib):
    from paper_2601_11553_amd.binding import Config
    ok = Config(1, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 1000, 1024)
    n = lib.percache_arena_bytes(ctypes.byref(ok))
    store = 2 * 16 * 8 * 512 * 128 * 2
    assert n >= store + 1000 * 1024 * 2 + 4096 * 64 * 8 and n % 256 == 0
    assert lib.percache_arena_bytes(None) == 0
    for field, bad in [("head_dim", 96), ("hidden", 1000), ("n_kv_heads", 3), ("slot_capacity", 100), ("emb_dim", 96),
                       ("n_layers", 0), ("rope_theta", 0.5)]:
        c = Config(1, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 1000, 1024)
        setattr(c, field, bad)
        assert lib.percache_arena_bytes(ctypes.byref(c)) == 0, field


def test_create_rejects_bad_arguments_without_touching_a_device(lib):
    from paper_2601_11553_amd.binding import Config
    out = ctypes.c_void_p()
    c = Config(1, 1024, 16, 8, 96, 16, 512, 4096, 10000.0, 0, 0)
    assert lib.percache_create(ctypes.byref(c), None, 0, ctypes.byref(out)) == -2
    assert b"head_dim" in lib.percache_last_error(None)
    c.head_dim = 128
    assert lib.percache_create(ctypes.byref(c), None, 0, ctypes.byref(out)) == -1      # NULL arena
    assert lib.percache_create(ctypes.byref(c), 0x1001, 1 << 40, ctypes.byref(out)) == -1  # misaligned
    assert lib.percache_create(ctypes.byref(c), 0x1000, 16, ctypes.byref(out)) == -5   # too small
    assert out.value is None
    assert lib.percache_bank_size(None) == -1
    assert lib.percache_kv_len(None, 0, 0) == -1
    lib.percache_destroy(None)


def test_arena_of_8_bit_slots_is_half_the_store_plus_scales(lib):
    from paper_2601_11553_amd.binding import Config
    c = Config(2, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 0, 0, 0)
    c8 = Config(2, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 0, 0, 1)
    a, a8 = lib.percache_arena_bytes(ctypes.byref(c)), lib.percache_arena_bytes(ctypes.byref(c8))
    store = 2 * 16 * 8 * 512 * 128          # elements of one store (K or V)
    scales = 2 * 16 * 8 * (512 // 64) * 4   # bytes
    assert a - a8 == 2 * store - 2 * scales
    bad = Config(2, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 0, 0, 2)
    assert lib.percache_arena_bytes(ctypes.byref(bad)) == 0


def test_arena_of_a_store_with_both_slot_formats(lib):
    from paper_2601_11553_amd.binding import Config
    base = Config(2, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 0, 0, 0, 0)
    mixed = Config(2, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 0, 0, 0, 6)
    a, m = lib.percache_arena_bytes(ctypes.byref(base)), lib.percache_arena_bytes(ctypes.byref(mixed))
    per_slot = 2 * 8 * 512 * 128            # elements of one slot over both layers (K or V)
    scales = 2 * 6 * 8 * (512 // 64) * 4    # bytes
    assert a - m == 2 * 6 * per_slot - 2 * scales   # six slots shrink from 2 bytes to 1 byte per element, plus their scales
    all8 = Config(2, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 0, 0, 0, 16)
    flag = Config(2, 1024, 16, 8, 128, 16, 512, 4096, 10000.0, 0, 0, 1, 0)
    assert lib.percache_arena_bytes(ctypes.byref(all8)) == lib.percache_arena_bytes(ctypes.byref(flag))
