"""Seeded random sweeps over the argument space of the main entry points, each case against
the oracle: sizes with ragged tails, group sizes that are not powers of two, every element
format and width; and, for the fused weight gradient, groups that straddle the tiles of k."""
import numpy as np
import pytest
import torch

from daf_inputs import BF16, F16, F32, Workload, to_numpy_bits, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import hip_harness
    assert torch.cuda.is_available()
    return hip_harness


@pytest.mark.parametrize("seed", range(6))
def test_quantize_dequantize_random_cases(H, seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(12):
        dtype = int(rng.choice([F32, F16, BF16]))
        gs = int(rng.choice([32, 64, 96, 128, 160, 256, 288, 512, 1024, 4096, 4128, 8192]))
        n = int(rng.integers(1, 9)) * gs * int(rng.integers(1, 40)) + int(rng.integers(0, gs))
        n = max(n, 1)
        G = (n + gs - 1) // gs
        kind = int(rng.integers(0, 5))
        bits = (rng.choice([1, 2, 4, 8], G).astype(np.uint8) if kind == 4 else np.array([[1, 2, 4, 8][kind]], np.uint8))
        g = torch.Generator().manual_seed(int(rng.integers(0, 1 << 30)))
        x = (torch.randn(n, generator=g) * float(np.exp(rng.normal(0, 3)))).to(torch_dtype(dtype))
        x[torch.isinf(x.float())] = 0
        w = Workload(f"sweep{seed}_{case}_dt{dtype}_gs{gs}_n{n}_k{kind}", x, dtype, gs, bits, int(rng.integers(0, 1 << 40)))
        print("case", w.name, flush=True)
        H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.parametrize("case", [(64, 256, 960, 96, "mixed", BF16), (96, 256, 960, 160, 4, F16), (64, 320, 960, 192, "mixed", F32),
                                  (128, 256, 384, 96, "mixed", BF16), (64, 256, 1152, 288, 2, F32), (32, 4096, 4608, 96, "mixed", BF16),
                                  (160, 256, 768, 384, "mixed", F16), (64, 256, 2048, 1024, 8, BF16)])
def test_grad_weight_groups_that_straddle_tiles(case):
    """Group sizes that are not powers of two (and groups wider than a tile of k): a tile row then
    reads two to four groups, or a part of one."""
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    from tests.test_gpu_unpack_matmul import _case
    M, N, K, gs, bits, dtype = case
    print("case straddle", case, flush=True)
    _case(daf, orc, M, N, K, gs, bits, dtype, 31)


@pytest.mark.parametrize("seed", range(4))
def test_list_calls_random_lists(seed):
    """Random lists of up to 40 tensors (more than one launch's 32 descriptors) of one format:
    sizes from one element to a few tiles, any group size and width kind in any order."""
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    from tests.test_gpu_batch import _roundtrip
    rng = np.random.default_rng(2000 + seed)
    dtype = [F32, F16, BF16, F32][seed]
    specs = []
    for _ in range(int(rng.integers(3, 41))):
        gs = int(rng.choice([32, 64, 96, 128, 256, 1024, 4096, 8192]))
        n = int(rng.integers(1, 4)) * gs * int(rng.integers(1, 12)) + int(rng.integers(0, gs))
        specs.append((n, gs, [1, 2, 4, 8, "mixed"][int(rng.integers(0, 5))]))
    _roundtrip(daf, orc, dtype, specs)


@pytest.mark.parametrize("seed", range(4))
def test_fused_relu_random_cases(seed):
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    from tests.test_gpu_fused_relu import _check, _run
    rng = np.random.default_rng(3000 + seed)
    for case in range(8):
        dtype = int(rng.choice([F32, F16, BF16]))
        gs = int(rng.choice([32, 64, 96, 128, 256, 1024, 4096]))
        n = int(rng.integers(1, 6)) * gs * int(rng.integers(1, 30)) + int(rng.integers(0, gs))
        G = (n + gs - 1) // gs
        kind = int(rng.integers(0, 5))
        b = rng.choice([1, 2, 4, 8], G).astype(np.uint8) if kind == 4 else np.array([[1, 2, 4, 8][kind]], np.uint8)
        g = torch.Generator().manual_seed(int(rng.integers(0, 1 << 30)))
        z = torch.randn(n, generator=g).to(torch_dtype(dtype))
        plan = daf.daf_plan((n,), gs, torch.from_numpy(b).cuda() if b.size > 1 else int(b[0]))
        sd = int(rng.integers(0, 1 << 40))
        in_place = bool(rng.integers(0, 2))
        print("case relu sweep", seed, case, dtype, gs, n, kind, in_place, flush=True)
        _check(orc, z, dtype, gs, b, sd, _run(daf, plan, z.clone(), sd, in_place))
        plan.destroy()


@pytest.mark.parametrize("seed", range(6))
def test_any_group_size_random_cases(H, seed):
    """Group sizes drawn from every regime of the dispatch (32 * m for m around 1 ... 2200, with
    extra weight on the borders between the kernels), random lengths with and without whole
    last groups: quantize + dequantize against the oracle, and the statistics-only call."""
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    rng = np.random.default_rng(3000 + seed)
    borders = [1, 2, 3, 4, 5, 63, 64, 65, 127, 128, 129, 130, 255, 256, 257, 384, 511, 512, 513, 1023, 1024, 1025, 1030, 2047,
               2048, 2049]
    for case in range(14):
        m = int(rng.choice(borders)) if rng.random() < 0.5 else int(rng.integers(1, 2200))
        gs = 32 * m
        groups = int(rng.integers(1, max(2, 300000 // gs)))
        n = groups * gs + (int(rng.integers(1, gs)) if rng.random() < 0.6 else 0)
        dtype = int(rng.choice([F32, F16, BF16]))
        G = (n + gs - 1) // gs
        kind = int(rng.integers(0, 5))
        bits = (rng.choice([1, 2, 4, 8], G).astype(np.uint8) if kind == 4 else np.array([[1, 2, 4, 8][kind]], np.uint8))
        g = torch.Generator().manual_seed(int(rng.integers(0, 1 << 30)))
        x = (torch.randn(n, generator=g) * float(np.exp(rng.normal(0, 2)))).to(torch_dtype(dtype))
        x[torch.isinf(x.float())] = 0
        w = Workload(f"anygs{seed}_{case}_dt{dtype}_m{m}_n{n}_k{kind}", x, dtype, gs, bits, int(rng.integers(0, 1 << 40)))
        print("case", w.name, flush=True)
        res = H.run_hip(w)
        H.assert_full_parity(w, res)
        mn = torch.full((G,), float("nan"), device="cuda:0")
        mx = torch.full((G,), float("nan"), device="cuda:0")
        daf.daf_group_minmax(res.plan, x.cuda(), mn, mx)
        torch.cuda.synchronize()
        omn, omx = orc.group_minmax(to_numpy_bits(x), dtype, gs)
        assert np.array_equal(mn.cpu().numpy().view(np.uint32), omn.view(np.uint32)), w.name
        assert np.array_equal(mx.cpu().numpy().view(np.uint32), omx.view(np.uint32)), w.name
