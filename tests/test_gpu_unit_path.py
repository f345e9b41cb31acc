"""GPU parity for group sizes that are a multiple of 32 elements but not a power of two (rows
of a transformer activation: 768, 3072, ...), which the quantize call handles one wave per
run of whole groups: words, min, scale and the dequantized values must equal the oracle's,
bit for bit, for every element format and width, with groups left over after the last whole
tile, a short last group, constant groups and groups whose range is tiny."""
import numpy as np
import pytest
import torch

from daf_inputs import BF16, F16, F32, Workload, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import hip_harness
    assert torch.cuda.is_available(), "GPU tests need cuda:0"
    return hip_harness

# 32 * m elements: m = 3 (42 groups per tile), 5, 24 (ViT row), 49, 65 and 127 (one group per
# tile, half and almost full), 96 (3072), 128 is the power-of-two path's
GROUP_SIZES = [96, 160, 768, 1568, 2080, 3072, 4064]


def _workload(dtype, gs, bits, seed, tiles=3, extra_groups=2, last=17):
    k = 128 // (gs // 32)
    n = (tiles * k + extra_groups) * gs + last          # whole tiles, groups after them, a short last group
    G = (n + gs - 1) // gs
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(n, generator=g) * 4.0 + 0.5
    x[gs: 2 * gs] = 1.25                                  # a constant group
    x[2 * gs: 3 * gs] = 1.0 + torch.rand(gs, generator=g) * 1e-30   # constant after rounding, or a tiny range
    x = x.to(torch_dtype(dtype))
    b = (np.random.default_rng(seed).choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed"
         else np.array([bits], np.uint8))
    return Workload(f"unit_{dtype}_{gs}_{bits}", x, dtype, gs, b, 1000 + seed)


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("gs", GROUP_SIZES)
@pytest.mark.parametrize("bits", [1, 2, 4, 8, "mixed"])
def test_unit_path_matrix(H, dtype, gs, bits):
    w = _workload(dtype, gs, bits, seed=gs + 7 * dtype)
    print("case", w.name, w.numel, flush=True)
    H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("gs,tiles", [(96, 1), (96, 40), (768, 1), (768, 129), (3072, 33), (4064, 5)])
def test_unit_path_tile_counts(H, dtype, gs, tiles):
    """One tile (a single wave), and counts that do not fill the last workgroup."""
    for extra, last in ((0, 0), (0, 5), (1, 0)):
        w = _workload(dtype, gs, "mixed", seed=tiles + extra + last, tiles=tiles, extra_groups=extra, last=last)
        print("case", w.name, tiles, extra, last, flush=True)
        H.assert_full_parity(w, H.run_hip(w))


def test_unit_path_every_m(H):
    """Every group size 32 * m, 3 <= m <= 128: the unit-to-group division and the sharing of a
    group's units among lanes are exact for each."""
    for m in range(3, 129):
        gs = 32 * m
        w = _workload(BF16 if m % 2 else F32, gs, "mixed" if m % 3 else 2, seed=m, tiles=2, extra_groups=1, last=3)
        if m % 16 == 3:
            print("case", w.name, flush=True)
        H.assert_full_parity(w, H.run_hip(w))


def test_unit_path_extreme_values(H):
    """Largest finite magnitudes of both signs in one group (the reciprocal of the range
    underflows to a subnormal) and a subnormal range (the reciprocal overflows)."""
    gs = 768
    for dtype in (F32, F16, BF16):
        w = _workload(dtype, gs, 4, seed=5)
        big = torch.finfo(torch_dtype(dtype)).max
        x = w.x.clone()
        x[4 * gs] = big / 2
        x[4 * gs + 1] = -big / 2
        tiny = torch.finfo(torch_dtype(dtype)).tiny
        x[5 * gs: 6 * gs] = 0.0
        x[5 * gs + 3] = tiny / 4 if dtype != BF16 else tiny
        w.x = x
        H.assert_full_parity(w, H.run_hip(w))


# ---- groups of 4128 .. 65536 elements: one workgroup per group ---------------------------------

def _long_workload(dtype, gs, bits, seed, groups, last):
    n = groups * gs + last
    G = (n + gs - 1) // gs
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(n, generator=g) * 2.0 - 0.25
    if groups > 1:
        x[gs: 2 * gs] = -3.5                              # a constant group
    x = x.to(torch_dtype(dtype))
    b = (np.random.default_rng(seed).choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed"
         else np.array([bits], np.uint8))
    return Workload(f"long_{dtype}_{gs}_{bits}", x, dtype, gs, b, 2000 + seed)


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("gs", [4128, 5120, 11008, 12320, 32736, 40000, 65504])   # 129 ... 2047 units: 2, 2, 3, 4, 8, 10, 16 waves
@pytest.mark.parametrize("bits", [1, 2, 4, 8, "mixed"])
def test_long_groups_not_a_multiple_of_the_tile(H, dtype, gs, bits):
    w = _long_workload(dtype, gs, bits, seed=gs % 1000 + dtype, groups=5, last=gs // 3 + 1)
    print("case", w.name, w.numel, flush=True)
    H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.parametrize("dtype,gs,bits", [(F32, 8192, 2), (BF16, 8192, "mixed"), (F16, 16384, 4), (F32, 32768, "mixed"),
                                           (BF16, 65536, 2), (F16, 49152, "mixed")])
def test_long_groups_of_whole_tiles(H, dtype, gs, bits):
    """256 groups or more: the one-workgroup-per-group kernel also takes groups that are a whole
    number of tiles (fewer groups go through the two-pass route, tested elsewhere)."""
    w = _long_workload(dtype, gs, bits, seed=gs % 999, groups=257, last=100)
    print("case", w.name, w.numel, flush=True)
    H.assert_full_parity(w, H.run_hip(w))


def test_long_groups_every_wave_count(H):
    """Group sizes around every change of the number of waves and of the slice length."""
    for m in (129, 130, 255, 256 + 1, 383, 384, 385, 511, 513, 640, 767, 769, 896, 897, 1000, 1024, 1025, 1153, 1536, 1921, 2047):
        gs = 32 * m
        if m == 1024:
            continue                                     # a power of two: whole tiles, covered above
        w = _long_workload(BF16 if m % 2 else F32, gs, "mixed" if m % 3 else 8, seed=m, groups=3, last=0)
        print("case", w.name, flush=True)
        H.assert_full_parity(w, H.run_hip(w))


def test_group_minmax_every_m(H):
    """daf_group_minmax on every group size 32 * m, 3 <= m <= 128, and on long groups, against
    the oracle's per-group minimum and maximum."""
    import paper_2507_07149_amd as daf
    from daf_inputs import to_numpy_bits
    from oracle import daf_oracle as orc
    for m in list(range(3, 129)) + [129, 344, 385, 1023, 1500]:
        gs = 32 * m
        dtype = (F32, F16, BF16)[m % 3]
        n = (2 * max(1, 128 // m) + 1) * gs + (m % 5) * 7
        g = torch.Generator().manual_seed(m)
        x = (torch.randn(n, generator=g) * 3).to(torch_dtype(dtype))
        plan = daf.daf_plan((n,), gs, 8)
        G = plan.num_groups
        mn = torch.full((G,), float("nan"), device="cuda:0")
        mx = torch.full((G,), float("nan"), device="cuda:0")
        daf.daf_group_minmax(plan, x.cuda(), mn, mx)
        torch.cuda.synchronize()
        omn, omx = orc.group_minmax(to_numpy_bits(x), dtype, gs)
        assert np.array_equal(mn.cpu().numpy().view(np.uint32), omn.view(np.uint32)), f"min, m={m}"
        assert np.array_equal(mx.cpu().numpy().view(np.uint32), omx.view(np.uint32)), f"max, m={m}"
        plan.destroy()


def test_quantize_routes(H):
    """daf_plan_quantize_route names the kernels the parity tests above exercise."""
    import paper_2507_07149_amd as daf
    cases = [((4096 * 8,), 256, 2, torch.float32, "tile"), ((768 * 50,), 768, 2, torch.bfloat16, "units"),
             ((11008 * 5,), 11008, 2, torch.float16, "long"), ((8192 * 300,), 8192, 2, torch.float32, "long"),
             ((8192 * 5,), 8192, 2, torch.float32, "two_pass"), ((65536 * 300,), 65536, 2, torch.float32, "long"),
             ((131072 * 300,), 131072, 2, torch.float32, "two_pass"),
             ((100000,), 100000 // 32 * 32 + 32, 2, torch.float32, "two_pass"),          # one group for the tensor
             ((40000 * 4,), 40000, 2, torch.float32, "long"), ((69984 * 4,), 69984, 2, torch.float32, "group")]
    for shape, gs, bits, dt, want in cases:
        p = daf.daf_plan(shape, gs, bits)
        assert p.quantize_route(dt) == want, (shape, gs, want)
        p.destroy()
    b = torch.from_numpy(np.random.default_rng(0).choice([1, 2, 4, 8], 50).astype(np.uint8)).cuda()
    p = daf.daf_plan((768 * 50,), 768, b)
    assert p.quantize_route(torch.float32) == "units"
    p.destroy()
