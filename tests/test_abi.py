"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2507_07149_amd as daf
    return daf.load_library()


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if header.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, header)).read(), flags=re.S)
            names |= set(re.findall(r"\b(daf_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"daf_plan", "daf_quantize_pack", "daf_unpack_dequantize", "daf_plan_destroy", "daf_store_create"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in include/*.h but not exported"


def test_python_binding_has_the_same_entry_points():
    import paper_2507_07149_amd as daf
    for name in ("daf_plan", "daf_quantize_pack", "daf_unpack_dequantize"):
        assert callable(getattr(daf, name))


def test_rand_bits_and_status_strings(lib):
    assert lib.daf_rand_bits() == 8
    for code in (0, -1, -2, -3, -4, 77):
        assert lib.daf_status_string(code)


def _plan(lib, shape, gs, bits):
    shp = (ctypes.c_int64 * len(shape))(*shape)
    b = (ctypes.c_uint8 * len(bits))(*bits)
    out = ctypes.c_void_p()
    rc = lib.daf_plan(shp, len(shape), gs, ctypes.cast(b, ctypes.c_void_p), len(bits), None, ctypes.byref(out))
    return rc, out


def test_uniform_plan_needs_no_device(lib):
    rc, p = _plan(lib, (64, 256, 56, 56), 256, [2])
    assert rc == 0
    assert lib.daf_plan_packed_words(p) == 3211264
    assert lib.daf_plan_num_groups(p) == 200704
    assert lib.daf_plan_num_elements(p) == 51380224
    assert lib.daf_plan_group_size(p) == 256 and lib.daf_plan_uniform_bits(p) == 2
    lib.daf_plan_destroy(p)
    rc, p = _plan(lib, (37,), 32, [4])                 # short last group: 4 + 1 words
    assert rc == 0 and lib.daf_plan_packed_words(p) == 5
    off = (ctypes.c_uint32 * 2)()
    assert lib.daf_plan_copy_offsets(p, off) == 0 and list(off) == [0, 4]
    assert lib.daf_plan_set_output_cached(p, 1) == 0 and lib.daf_plan_set_output_cached(p, 0) == 0
    assert lib.daf_plan_set_output_cached(p, 2) == -1 and lib.daf_plan_set_output_cached(p, -1) == -1
    assert lib.daf_plan_set_output_cached(None, 1) == -1
    lib.daf_plan_destroy(p)
    lib.daf_plan_destroy(None)


@pytest.mark.parametrize("shape,gs,bits,want", [
    ((64,), 32, [3], -1), ((64,), 32, [0], -1), ((64,), 32, [16], -1),
    ((64,), 48, [2], -2), ((64,), 0, [2], -2), ((64,), 16, [2], -2),
    ((0,), 32, [2], -1), ((4, -1), 32, [2], -1),
    ((64,), 32, [2, 2, 2], -1),                        # neither 1 nor G widths
    ((1 << 40,), 32, [8], -2),                         # 2^38 words
])
def test_plan_argument_errors(lib, shape, gs, bits, want):
    rc, p = _plan(lib, shape, gs, bits)
    assert rc == want and not p.value


def test_null_arguments(lib):
    out = ctypes.c_void_p()
    assert lib.daf_plan(None, 1, 32, None, 1, None, ctypes.byref(out)) == -1
    shp = (ctypes.c_int64 * 1)(64)
    assert lib.daf_plan(shp, 0, 32, ctypes.cast(shp, ctypes.c_void_p), 1, None, ctypes.byref(out)) == -1
    rc, p = _plan(lib, (64,), 32, [2])
    assert lib.daf_quantize_pack(p, None, 0, 0, None, None, None, None) == -1
    assert lib.daf_unpack_dequantize(p, None, None, None, None, None, 0, None) == -1
    assert lib.daf_quantize_pack(None, 16, 0, 0, 16, 16, 16, None) == -1
    # misaligned x and unknown dtype are rejected before any launch
    assert lib.daf_quantize_pack(p, 20, 0, 0, 16, 16, 16, None) == -1
    assert lib.daf_quantize_pack(p, 16, 7, 0, 16, 16, 16, None) == -2
    assert lib.daf_unpack_dequantize(p, 16, 16, 16, None, 16, 9, None) == -2
    lib.daf_plan_destroy(p)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2507_07149_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libdaf.so"))
    with pytest.raises(ImportError):
        binding.load_library()


@pytest.mark.parametrize("n,gs,dtype,want", [
    (4096 * 10, 256, 0, 0), (4096 * 10, 4096, 2, 0), (4096 * 10, 32, 1, 0),         # tile
    (768 * 100, 768, 0, 1), (96 * 1000, 96, 1, 1), (4064 * 9, 4064, 2, 1),          # units
    (11008 * 7, 11008, 0, 2), (4128 * 3, 4128, 2, 2), (32736 * 2 + 5, 32736, 1, 2),  # long (not whole tiles)
    (40000 * 3, 40000, 0, 2), (65504 * 2, 65504, 2, 2),                              # long, up to 65536
    (69984 * 3, 69984, 0, 4), (65568 * 2, 65568, 2, 4),                              # group by group
    (100, 256, 0, 4), (700, 768, 1, 4),                                              # no whole group
])
def test_quantize_route_of_uniform_plans(lib, n, gs, dtype, want):
    """The route a plan's quantize call takes, for plans that need no device (one width, no
    statistics pass): tile, units, long, group by group."""
    rc, p = _plan(lib, (n,), gs, [2])
    assert rc == 0
    assert lib.daf_plan_quantize_route(p, dtype) == want
    assert lib.daf_plan_quantize_route(p, 7) == -2 and lib.daf_plan_quantize_route(None, 0) == -1
    lib.daf_plan_destroy(p)
