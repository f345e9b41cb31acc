"""GPU parity of the producer fusion into a matrix product: daf_linear_quantize_pack(x, W) must
write y = x W^T rounded to the element format and the words, min and scale that the oracle's
quantize_pack gives for that y.

Bit-exact cases use small-integer operands (multiples of 1/4), for which every partial sum is
exact in binary32 in any order, so the oracle's product (double precision, rounded once) and the
kernel's (binary32 accumulation on the matrix cores) are the same numbers.  For normal random
operands the order of the additions shows in the last place of y, so y is compared with a
tolerance derived from the accumulation, and the packed output is checked through properties
that hold for any y: min and scale are Eq. 1 of the y the kernel wrote, and the codes are within
one step of it."""
import numpy as np
import pytest
import torch

from daf_inputs import BF16, F16, to_numpy_bits, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    assert torch.cuda.is_available()
    return daf, orc


def _bits_for(rng, G, bits):
    return rng.choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed" else np.array([bits], np.uint8)


def _run(daf, x, w, gs, b, seed):
    M, K = x.shape
    N = w.shape[0]
    plan = daf.daf_plan((M, N), gs, torch.from_numpy(b).cuda() if b.size > 1 else int(b[0]))
    G = plan.num_groups
    y = torch.full((M, N), 7.0, dtype=x.dtype, device="cuda:0")
    words = torch.full((plan.packed_words,), -1, dtype=torch.int32, device="cuda:0")
    mn = torch.full((G,), float("nan"), device="cuda:0")
    sc = torch.full((G,), float("nan"), device="cuda:0")
    daf.daf_linear_quantize_pack(plan, x.cuda(), w.cuda(), seed, y, words, mn, sc)
    torch.cuda.synchronize()
    plan.destroy()
    return y.cpu(), words.cpu().numpy().view(np.uint32), mn.cpu().numpy(), sc.cpu().numpy()


def _integer_operands(rng, M, N, K, dtype):
    x = torch.from_numpy(rng.integers(-3, 4, (M, K)).astype(np.float32)).to(torch_dtype(dtype))
    w = torch.from_numpy(rng.integers(-3, 4, (N, K)).astype(np.float32) / 4).to(torch_dtype(dtype))
    return x, w


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("gs", [32, 64, 128])
@pytest.mark.parametrize("bits", [1, 2, 4, 8, "mixed"])
def test_linear_quantize_pack_bit_exact_on_exact_products(env, dtype, gs, bits):
    daf, orc = env
    M, N, K = 512, 768, 192                     # 2 x 3 tiles, three steps of 64 along k
    rng = np.random.default_rng(1000 * gs + dtype)
    x, w = _integer_operands(rng, M, N, K, dtype)
    b = _bits_for(rng, M * N // gs, bits)
    print("case", dtype, gs, bits, flush=True)
    y, words, mn, sc = _run(daf, x, w, gs, b, 77)
    oy = orc.linear_forward(to_numpy_bits(x), to_numpy_bits(w), M, K, N, dtype)
    assert np.array_equal(to_numpy_bits(y).view(oy.dtype).reshape(-1), oy), "y differs from the rounded product"
    ow, omn, osc, _ = orc.quantize_pack(oy, dtype, gs, b, 77)
    assert np.array_equal(words, ow), "packed words differ"
    assert np.array_equal(mn.view(np.uint32), omn.view(np.uint32)), "min differs"
    assert np.array_equal(sc.view(np.uint32), osc.view(np.uint32)), "scale differs"


@pytest.mark.parametrize("shape", [(256, 256, 64), (256, 1024, 4096), (1024, 256, 128), (2048, 2816, 512)])
def test_linear_quantize_pack_shapes(env, shape):
    """One step, many steps, more tiles than compute-unit dies (the tile order is remapped when the
    tile count is a multiple of 8), a tile count that is not."""
    daf, orc = env
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    x, w = _integer_operands(rng, M, N, K, BF16)
    b = _bits_for(rng, M * N // 64, "mixed")
    print("case", shape, flush=True)
    y, words, mn, sc = _run(daf, x, w, 64, b, 5)
    oy = orc.linear_forward(to_numpy_bits(x), to_numpy_bits(w), M, K, N, BF16)
    assert np.array_equal(to_numpy_bits(y).view(oy.dtype).reshape(-1), oy)
    ow, omn, osc, _ = orc.quantize_pack(oy, BF16, 64, b, 5)
    assert np.array_equal(words, ow) and np.array_equal(mn.view(np.uint32), omn.view(np.uint32))
    assert np.array_equal(sc.view(np.uint32), osc.view(np.uint32))


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_linear_quantize_pack_normal_operands(env, dtype):
    daf, orc = env
    M, N, K = 512, 512, 1024
    g = torch.Generator().manual_seed(9)
    x = torch.randn(M, K, generator=g).to(torch_dtype(dtype))
    w = (torch.randn(N, K, generator=g) / 32).to(torch_dtype(dtype))
    gs = 64
    b = _bits_for(np.random.default_rng(3), M * N // gs, "mixed")
    y, words, mn, sc = _run(daf, x, w, gs, b, 21)
    # y against the double-precision product: half a unit in the last place of the format for the
    # rounding, plus the error of K binary32 additions (each below 2^-24 of the sum of magnitudes)
    xd, wd = x.double().numpy(), w.double().numpy()
    exact = xd @ wd.T
    yd = y.double().numpy()
    half_ulp = 2.0 ** (-11 if dtype == F16 else -8)
    tol = np.abs(exact) * half_ulp * 1.001 + (np.abs(xd) @ np.abs(wd).T) * (K + 2) * 2.0 ** -24 + 1e-30
    assert np.all(np.abs(yd - exact) <= tol), float(np.max(np.abs(yd - exact) / tol))
    # the packed output against the y the kernel wrote: Eq. 1 on it, and codes within one step
    yf = y.float().numpy().reshape(-1, gs)
    assert np.array_equal(mn, yf.min(axis=1) + 0.0)
    L = ((1 << b.astype(np.int64)) - 1).astype(np.float32)
    assert np.array_equal(sc, ((yf.max(axis=1) + np.float32(0)) - (yf.min(axis=1) + np.float32(0))) / L)
    xh = orc.widen(orc.unpack_dequantize(words, mn, sc, b, M * N, gs, dtype)[0], dtype).reshape(-1, gs)
    step = sc[:, None] * 1.01 + np.abs(yf) * 2 * half_ulp + 1e-30
    assert np.all(np.abs(xh - yf) <= step)


def test_linear_quantize_pack_argument_errors(env):
    daf, orc = env
    x = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda:0")
    w = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda:0")
    y = torch.zeros(256, 256, dtype=torch.bfloat16, device="cuda:0")
    mk = lambda gs: daf.daf_plan((256, 256), gs, 4)
    def call(plan, x=x, w=w, y=y):
        words = torch.zeros(plan.packed_words, dtype=torch.int32, device="cuda:0")
        mn = torch.zeros(plan.num_groups, device="cuda:0")
        daf.daf_linear_quantize_pack(plan, x, w, 1, y, words, mn, mn.clone())
    call(mk(64))
    with pytest.raises(daf.DafError):          # group size the epilogue does not cover
        call(mk(256))
    with pytest.raises(daf.DafError):          # K not a multiple of 64
        call(mk(64), x=torch.zeros(256, 96, dtype=torch.bfloat16, device="cuda:0"),
             w=torch.zeros(256, 96, dtype=torch.bfloat16, device="cuda:0"))
    with pytest.raises(ValueError):            # the plan does not describe y
        call(daf.daf_plan((256, 512), 64, 4))
    with pytest.raises(ValueError):            # inner dimensions differ
        call(mk(64), w=torch.zeros(256, 128, dtype=torch.bfloat16, device="cuda:0"))
    with pytest.raises(daf.DafError):          # binary32 is not offered
        p = mk(64)
        words = torch.zeros(p.packed_words, dtype=torch.int32, device="cuda:0")
        mn = torch.zeros(p.num_groups, device="cuda:0")
        daf.daf_linear_quantize_pack(p, x.float(), w.float(), 1, y.float(), words, mn, mn.clone())
    torch.cuda.synchronize()
