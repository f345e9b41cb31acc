"""GPU parity of daf_minmax (both reduction methods) against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

from daf_inputs import BF16, F16, F32, make_config, to_numpy_bits, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    assert torch.cuda.is_available()
    ws = daf.daf_minmax_workspace()
    torch.cuda.synchronize()
    return daf, orc, ws


def _check(env, x: torch.Tensor, dtype: int):
    daf, orc, ws = env
    want = orc.minmax(to_numpy_bits(x), dtype)
    xd = x.cuda()
    for method in (daf.REDUCE_TWO_PASS, daf.REDUCE_ATOMIC, daf.REDUCE_ATOMIC, daf.REDUCE_TWO_PASS):
        out = torch.full((2,), float("nan"), device="cuda:0")
        daf.daf_minmax(xd, method, ws, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (method, got, want, x.numel())


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("n", [1, 3, 4, 5, 7, 8, 9, 255, 1000, 4099, 50_176, 393_216, 3_000_001])
def test_sizes_including_the_papers_shapes(env, dtype, n):
    """50,176 = [1,256,14,14] and 393,216 = [1,512,768] are the inputs of the paper's reduction
    experiment (Fig. 12)."""
    g = torch.Generator().manual_seed(n)
    x = (torch.randn(n, generator=g) * 3).to(torch_dtype(dtype))
    print("case", dtype, n, flush=True)
    _check(env, x, dtype)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_extremes_anywhere(env, dtype):
    n = 1_000_003
    g = torch.Generator().manual_seed(5)
    base = torch.randn(n, generator=g)
    for pos_min, pos_max in ((0, n - 1), (n - 1, 0), (n - 2, n // 2), (12345, n - 3), (n // 3, 7)):
        x = base.clone()
        x[pos_min] = -100.0
        x[pos_max] = 200.0
        _check(env, x.to(torch_dtype(dtype)), dtype)


def test_zero_and_negative_only(env):
    z = torch.zeros(5000)
    z[::2] = -0.0
    _check(env, z, F32)
    _check(env, -torch.rand(70_001) - 1, F32)
    _check(env, torch.full((129,), 2.5), F32)


def test_resnet50_activation(env):
    (w,) = make_config(2)
    _check(env, w.x.reshape(-1), w.dtype)


def test_argument_errors(env):
    daf, _, ws = env
    x = torch.zeros(1024, device="cuda:0")
    out = torch.zeros(2, device="cuda:0")
    with pytest.raises(daf.DafError) as e:
        daf.daf_minmax(x[1:], daf.REDUCE_ATOMIC, ws, out)          # misaligned
    assert e.value.status == -1
    with pytest.raises(daf.DafError):
        daf.daf_minmax(x, 7, ws, out)                              # unknown method
