"""The Python binding refuses tensors the kernels would read or write out of bounds (the C ABI
takes bare pointers and cannot see sizes).  Runs without a GPU: a uniform-width plan needs no
device, and every check fires before the foreign call."""
import pytest
import torch

import paper_2507_07149_amd as daf


@pytest.fixture()
def plan():
    p = daf.daf_plan((4, 1024), 256, 2)          # 4096 elements, 16 groups, 256 words
    yield p
    p.destroy()


def _bufs(plan, dtype=torch.float32):
    return (torch.zeros(plan.num_elements, dtype=dtype), torch.zeros(plan.packed_words, dtype=torch.int32),
            torch.zeros(plan.num_groups), torch.zeros(plan.num_groups))


def test_plan_caches_its_sizes(plan):
    assert (plan.num_elements, plan.num_groups, plan.packed_words, plan.group_size, plan.uniform_bits) == \
        (4096, 16, 256, 256, 2)


def test_right_sizes_on_the_host_are_refused_as_host_tensors(plan):
    x, words, mn, sc = _bufs(plan)
    with pytest.raises(ValueError, match="device"):
        daf.daf_quantize_pack(plan, x, 0, words, mn, sc)
    with pytest.raises(ValueError, match="device"):
        daf.daf_unpack_dequantize(plan, words, mn, sc, x)


@pytest.mark.parametrize("which,make,msg", [
    ("x", lambda p: torch.zeros(p.num_elements - 1), "elements"),
    ("x", lambda p: torch.zeros(p.num_elements + 4), "elements"),
    ("x", lambda p: torch.zeros(p.num_elements, dtype=torch.float64), "dtype"),
    ("x", lambda p: torch.zeros(2 * p.num_elements)[::2], "contiguous"),
    ("words", lambda p: torch.zeros(p.packed_words - 1, dtype=torch.int32), "out_words"),
    ("words", lambda p: torch.zeros(p.packed_words, dtype=torch.int64), "dtype"),
    ("mn", lambda p: torch.zeros(p.num_groups - 1), "out_min"),
    ("sc", lambda p: torch.zeros(p.num_groups, dtype=torch.float16), "out_scale"),
    ("x", lambda p: [0.0] * p.num_elements, "torch.Tensor"),
])
def test_quantize_pack_rejects(plan, which, make, msg):
    args = dict(zip(("x", "words", "mn", "sc"), _bufs(plan)))
    args[which] = make(plan)
    with pytest.raises(ValueError, match=msg):
        daf.daf_quantize_pack(plan, args["x"], 0, args["words"], args["mn"], args["sc"])


def test_unpack_dequantize_rejects(plan):
    x, words, mn, sc = _bufs(plan, torch.bfloat16)
    with pytest.raises(ValueError, match="words"):
        daf.daf_unpack_dequantize(plan, words[:-1], mn, sc, x)
    with pytest.raises(ValueError, match="out_x"):
        daf.daf_unpack_dequantize(plan, words, mn, sc, x[:-8])
    with pytest.raises(ValueError, match="bits"):
        daf.daf_unpack_dequantize(plan, words, mn, sc, x, bits=torch.zeros(plan.num_groups - 1, dtype=torch.uint8))
    with pytest.raises(ValueError, match="scale"):
        daf.daf_unpack_dequantize(plan, words, mn, sc[:3], x)


def test_list_calls_and_fused_calls_reject(plan):
    x, words, mn, sc = _bufs(plan)
    with pytest.raises(ValueError, match="elements"):
        daf.quantize_items([(plan, x[:100], 0, words, mn, sc)])
    with pytest.raises(ValueError, match="out_x"):
        daf.dequantize_items([(plan, words, mn, sc, x[:100], None)])
    with pytest.raises(ValueError, match="out_metrics"):
        daf.daf_quantize_pack_metrics(plan, x, 0, words, mn, sc, torch.zeros(3 * plan.num_groups - 1))
    with pytest.raises(ValueError, match="out_y"):
        daf.daf_relu_quantize_pack(plan, x, 0, x[:-4], words, mn, sc)
    with pytest.raises(ValueError, match="out_grad_z"):
        daf.daf_unpack_relu_backward(plan, words, mn, sc, x, x.half())
    with pytest.raises(ValueError, match="out_max"):
        daf.daf_group_minmax(plan, x, mn, sc[:-1])
    with pytest.raises(ValueError, match="grad_y"):
        daf.daf_unpack_matmul_grad_weight(plan, words, mn, sc, torch.zeros(4, 63), torch.zeros(64, 1024))
    with pytest.raises(ValueError, match="out_bits"):
        daf.daf_select_bits(mn, sc, (2, 4), torch.zeros(3, dtype=torch.uint8), torch.zeros(1 << 20, dtype=torch.uint8))
    with pytest.raises(ValueError, match="out_minmax"):
        daf.daf_minmax(x, daf.REDUCE_TWO_PASS, torch.zeros(1 << 16, dtype=torch.uint8), torch.zeros(1))


def test_linear_tile_map_visits_every_tile_once():
    """The workgroup -> output tile map of daf_linear_quantize_pack (a host copy of the kernel's)
    is a bijection for tile grids with and without whole rounds of 256 workgroups, whole panels
    of four tile rows, and for a single tile; and 32 consecutive workgroups of one die (every
    eighth index) stay inside a compact patch when the grid is large."""
    import ctypes
    from paper_2507_07149_amd.binding import load_library
    L = load_library()
    for tiles_m, tiles_n in ((1, 1), (2, 3), (4, 8), (8, 32), (128, 43), (7, 5), (3, 100), (9, 64), (128, 3)):
        seen = set()
        tm, tn = ctypes.c_int32(), ctypes.c_int32()
        for i in range(tiles_m * tiles_n):
            assert L.daf_linear_tile_of_workgroup(i, tiles_m, tiles_n, ctypes.byref(tm), ctypes.byref(tn)) == 0
            assert 0 <= tm.value < tiles_m and 0 <= tn.value < tiles_n
            seen.add((tm.value, tn.value))
        assert len(seen) == tiles_m * tiles_n, (tiles_m, tiles_n)
        assert L.daf_linear_tile_of_workgroup(tiles_m * tiles_n, tiles_m, tiles_n, ctypes.byref(tm), ctypes.byref(tn)) != 0
    tiles_m, tiles_n = 128, 43
    rows, cols = set(), set()
    tm, tn = ctypes.c_int32(), ctypes.c_int32()
    for s in range(32):                                   # die 3, first round
        L.daf_linear_tile_of_workgroup(8 * s + 3, tiles_m, tiles_n, ctypes.byref(tm), ctypes.byref(tn))
        rows.add(tm.value); cols.add(tn.value)
    assert len(rows) <= 4 and len(cols) <= 9
