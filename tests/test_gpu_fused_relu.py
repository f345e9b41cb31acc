"""GPU parity of the producer fusion: daf_relu_quantize_pack(z) must write y = max(z, +0) and
the same words, min and scale as the oracle's relu followed by its quantize_pack, bit for bit,
out of place and in place."""
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
    return daf, orc


def _run(daf, plan, z, seed, in_place):
    zd = z.cuda()
    y = zd if in_place else torch.full_like(zd, 7.0)
    G = plan.num_groups
    words = torch.full((max(plan.packed_words, 1),), -1, dtype=torch.int32, device="cuda:0")[: plan.packed_words]
    mn = torch.full((G,), float("nan"), device="cuda:0")
    sc = torch.full((G,), float("nan"), device="cuda:0")
    daf.daf_relu_quantize_pack(plan, zd, seed, y, words, mn, sc)
    torch.cuda.synchronize()
    if not in_place:
        assert torch.equal(zd.cpu().view(torch.int16 if z.element_size() == 2 else torch.int32),
                           z.view(torch.int16 if z.element_size() == 2 else torch.int32)), "the input was modified"
    return y.cpu(), words.cpu().numpy().view(np.uint32), mn.cpu().numpy(), sc.cpu().numpy()


def _check(orc, z, dtype, gs, b, seed, got):
    y, words, mn, sc = got
    oy = orc.relu(to_numpy_bits(z), dtype)
    ow, omn, osc, _ = orc.quantize_pack(oy, dtype, gs, b, seed)
    assert np.array_equal(to_numpy_bits(y).view(oy.dtype), oy), "y differs from max(z, +0)"
    assert np.array_equal(words, ow), "packed words differ"
    assert np.array_equal(mn.view(np.uint32), omn.view(np.uint32)), "min differs"
    assert np.array_equal(sc.view(np.uint32), osc.view(np.uint32)), "scale differs"


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("gs", [32, 64, 96, 128, 160, 256, 768, 1024, 2080, 3072, 4096, 4128, 11008])
@pytest.mark.parametrize("bits", [1, 2, 8, "mixed"])
@pytest.mark.parametrize("in_place", [False, True])
def test_fused_relu_matrix(env, dtype, gs, bits, in_place):
    daf, orc = env
    n = 4096 * 5 + 3 * gs + 21                      # several tiles, whole groups after them, a short last group
    G = (n + gs - 1) // gs
    g = torch.Generator().manual_seed(31 * gs + dtype)
    z = (torch.randn(n, generator=g) * 2.5).to(torch_dtype(dtype))
    z[::97] = 0.0
    z[5::193] = -0.0
    b = (np.random.default_rng(gs).choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed"
         else np.array([bits], np.uint8))
    print("case", dtype, gs, bits, in_place, flush=True)
    plan = daf.daf_plan((n,), gs, torch.from_numpy(b).cuda() if b.size > 1 else int(b[0]))
    _check(orc, z, dtype, gs, b, 11, _run(daf, plan, z, 11, in_place))
    plan.destroy()


def test_fused_relu_all_negative_and_tiny_inputs(env):
    daf, orc = env
    for dtype in (F32, F16, BF16):
        for n, gs in ((32, 32), (1, 32), (4096, 256), (8192 + 64, 64)):
            z = -torch.rand(n).abs().to(torch_dtype(dtype)) - 1.0          # everything becomes +0: constant groups
            plan = daf.daf_plan((n,), gs, 4)
            got = _run(daf, plan, z, 3, False)
            _check(orc, z, dtype, gs, np.array([4], np.uint8), 3, got)
            assert not got[0].any()
            plan.destroy()


@pytest.mark.timeout(300)
def test_fused_relu_full_size_resnet_activation(env):
    """The benchmark's ResNet-50-like tensor at full size, pre-activation = the workload's values
    with random signs; every value of y and every packed word is compared."""
    daf, orc = env
    (w,) = make_config(2, 1.0)
    g = torch.Generator().manual_seed(5)
    sign = torch.randint(0, 2, w.x.shape, generator=g, dtype=torch.int8).float().mul_(2).sub_(1)
    z = (w.x + 0.25).mul_(sign).reshape(-1)
    print("case full-size fused relu", z.numel(), flush=True)
    plan = daf.daf_plan((z.numel(),), w.group_size, 2)
    _check(orc, z, F32, w.group_size, np.array([2], np.uint8), w.seed, _run(daf, plan, z, w.seed, True))
    plan.destroy()


def test_fused_relu_argument_errors(env):
    daf, _ = env
    z = torch.zeros(8192, device="cuda:0")
    plan = daf.daf_plan((8192,), 256, 2)
    words = torch.empty(plan.packed_words, dtype=torch.int32, device="cuda:0")
    mn = torch.empty(plan.num_groups, device="cuda:0")
    sc = torch.empty_like(mn)
    big = torch.zeros(8192 + 1024, device="cuda:0")
    with pytest.raises(daf.DafError) as e:                          # partially overlapping output
        daf.daf_relu_quantize_pack(plan, big[:8192], 0, big[1024:], words, mn, sc)
    assert e.value.status == -1
    with pytest.raises(ValueError):
        daf.daf_relu_quantize_pack(plan, z, 0, torch.zeros(8192, dtype=torch.float16, device="cuda:0"), words, mn, sc)
    long_plan = daf.daf_plan((8192,), 8192, 2)
    with pytest.raises(daf.DafError) as e:
        daf.daf_relu_quantize_pack(long_plan, z, 0, z, words, mn[:1], sc[:1])
    assert e.value.status == -2


# ---- consumer side: backward of max(z, 0) straight from the packed words --------------------

@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("gs", [32, 64, 96, 256, 4096, 8192])
@pytest.mark.parametrize("bits", [1, 2, 4, 8, "mixed"])
@pytest.mark.parametrize("in_place", [False, True])
def test_unpack_relu_backward_matrix(env, dtype, gs, bits, in_place):
    daf, orc = env
    n = 256 * 8 * 8 * 2 + 5 * gs + 13               # two blocks of chunks, whole groups, a ragged tail
    G = (n + gs - 1) // gs
    g = torch.Generator().manual_seed(17 * gs + dtype)
    y = torch.relu(torch.randn(n, generator=g) * 1.5).to(torch_dtype(dtype))       # the saved activation
    gy = torch.randn(n, generator=g).to(torch_dtype(dtype))
    gy[::101] = -0.0
    b = (np.random.default_rng(gs).choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed"
         else np.array([bits], np.uint8))
    print("case", dtype, gs, bits, in_place, flush=True)
    ow, omn, osc, _ = orc.quantize_pack(to_numpy_bits(y), dtype, gs, b, 23)
    oxh, _ = orc.unpack_dequantize(ow, omn, osc, b, n, gs, dtype)
    want = orc.relu_backward(oxh, to_numpy_bits(gy), dtype)
    assert 0.05 < np.count_nonzero(want) / n < 0.95      # both branches are exercised

    dbits = torch.from_numpy(b).cuda() if b.size > 1 else None
    plan = daf.daf_plan((n,), gs, dbits if dbits is not None else int(b[0]))
    words = torch.from_numpy(ow.view(np.int32)).cuda()
    mn, sc = torch.from_numpy(omn).cuda(), torch.from_numpy(osc).cuda()
    gyd = gy.cuda()
    out = gyd if in_place else torch.full_like(gyd, 3.0)
    daf.daf_unpack_relu_backward(plan, words, mn, sc, gyd, out)
    torch.cuda.synchronize()
    got = to_numpy_bits(out.cpu())
    assert np.array_equal(got.view(want.dtype), want), "grad_z differs"
    if not in_place:
        assert np.array_equal(to_numpy_bits(gyd.cpu()), to_numpy_bits(gy)), "grad_y was modified"
    plan.destroy()


def test_unpack_relu_backward_equals_threshold_on_materialised_xhat(env):
    """Against the unfused GPU sequence: daf_unpack_dequantize, then torch's threshold backward."""
    daf, _ = env
    (w,) = make_config(3, 1 / 8)
    x = torch.relu(w.x.float()).to(w.x.dtype).reshape(-1).cuda()
    bits = torch.from_numpy(w.bits).cuda()
    plan = daf.daf_plan(tuple(w.x.shape), w.group_size, bits)
    words = torch.empty(plan.packed_words, dtype=torch.int32, device="cuda:0")
    mn = torch.empty(plan.num_groups, device="cuda:0")
    sc = torch.empty_like(mn)
    daf.daf_quantize_pack(plan, x, w.seed, words, mn, sc)
    xh = torch.empty_like(x)
    daf.daf_unpack_dequantize(plan, words, mn, sc, xh)
    gy = torch.randn(x.numel(), device="cuda:0").to(x.dtype)
    gz = torch.empty_like(gy)
    daf.daf_unpack_relu_backward(plan, words, mn, sc, gy, gz)
    torch.cuda.synchronize()
    want = torch.where(xh > 0, gy, torch.zeros_like(gy))
    assert torch.equal(gz.view(torch.int16), want.view(torch.int16))
    plan.destroy()


def test_unpack_relu_backward_argument_errors(env):
    daf, _ = env
    plan = daf.daf_plan((8192,), 256, 2)
    words = torch.zeros(plan.packed_words, dtype=torch.int32, device="cuda:0")
    mn = torch.zeros(plan.num_groups, device="cuda:0")
    big = torch.zeros(8192 + 1024, device="cuda:0")
    with pytest.raises(daf.DafError) as e:
        daf.daf_unpack_relu_backward(plan, words, mn, mn, big[:8192], big[1024:])
    assert e.value.status == -1
    with pytest.raises(ValueError):
        daf.daf_unpack_relu_backward(plan, words, mn, mn, big[:8192], torch.zeros(8192, dtype=torch.float16, device="cuda:0"))


@pytest.mark.parametrize("dtype,gs,bits", [(F32, 8192, 2), (BF16, 16384, "mixed"), (F16, 32768, 8), (BF16, 65536, 4)])
def test_fused_relu_long_groups_of_whole_tiles(env, dtype, gs, bits):
    """256 groups or more of 8192 ... 65536 elements are read once (one workgroup per group), so
    the fused max(z, 0) exists for them; fewer such groups go through two passes and are refused."""
    daf, orc = env
    n = 257 * gs + 321
    G = (n + gs - 1) // gs
    g = torch.Generator().manual_seed(gs + dtype)
    z = (torch.randn(n, generator=g) * 2.0).to(torch_dtype(dtype))
    b = (np.random.default_rng(gs).choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed"
         else np.array([bits], np.uint8))
    plan = daf.daf_plan((n,), gs, torch.from_numpy(b).cuda() if b.size > 1 else int(b[0]))
    for in_place in (False, True):
        _check(orc, z, dtype, gs, b, 17, _run(daf, plan, z, 17, in_place))
    plan.destroy()
    few = daf.daf_plan((gs * 3,), gs, 2)
    zz = torch.zeros(gs * 3, dtype=torch_dtype(dtype), device="cuda:0")
    with pytest.raises(daf.DafError) as e:
        daf.daf_relu_quantize_pack(few, zz, 0, zz, torch.empty(few.packed_words, dtype=torch.int32, device="cuda:0"),
                                   torch.empty(3, device="cuda:0"), torch.empty(3, device="cuda:0"))
    assert e.value.status == -2
    few.destroy()
