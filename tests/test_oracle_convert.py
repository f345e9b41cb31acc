"""Pins for the oracle's 16-bit conversions against numpy float16 and torch bfloat16."""
import numpy as np
import torch

from oracle import daf_oracle as orc


def test_widen_f16_all_patterns():
    h = np.arange(65536, dtype=np.uint16)
    got = orc.widen(h, orc.F16)
    want = h.view(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.all(np.isnan(got[np.isnan(want)]))


def test_widen_bf16_all_patterns():
    h = np.arange(65536, dtype=np.uint16)
    got = orc.widen(h, orc.BF16)
    want = torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).float().numpy()
    ok = ~np.isnan(want)
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok])


def _samples():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(200_000).astype(np.float32) * (10.0 ** rng.uniform(-9, 5, 200_000)).astype(np.float32)
    # every float32 that sits exactly between two 16-bit neighbours, plus neighbours of those
    h = np.arange(0, 0x7C00, dtype=np.uint16)
    mid16 = (h.view(np.float16).astype(np.float64) + (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)) / 2
    mid16 = mid16[np.isfinite(mid16)].astype(np.float32)
    bf = (np.arange(0x0001, 0x7F7F, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)
    midbf = ((bf[:-1] + bf[1:]) / 2).astype(np.float32)
    edge = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 70000.0, 2.0 ** -24, 2.0 ** -25,
                     2.0 ** -25 * 1.0000001, 6.1e-5, 5.96e-8, 3.3e38, -3.3e38, 1e-45], dtype=np.float32)
    allv = np.concatenate([a, mid16, np.nextafter(mid16, np.float32(0)), np.nextafter(mid16, np.float32(np.inf)),
                           midbf, np.nextafter(midbf, np.float32(0)), edge])
    return np.concatenate([allv, -allv])


def test_narrow_f16_matches_numpy():
    x = _samples()
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.narrow(x, orc.F16), want)


def test_narrow_bf16_matches_torch():
    x = _samples()
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.narrow(x, orc.BF16), want)


def test_relu_matches_torch_on_every_16_bit_pattern_and_on_floats():
    # pinned against torch.relu on the CPU (an independent implementation), every finite pattern
    import torch
    pats = np.arange(65536, dtype=np.uint16)
    for dt, tdt in ((orc.F16, torch.float16), (orc.BF16, torch.bfloat16)):
        t = torch.from_numpy(pats.view(np.int16).copy()).view(tdt)
        finite = torch.isfinite(t.float()).numpy()
        want = torch.relu(t.float()).to(tdt).view(torch.int16).numpy().view(np.uint16)
        got = orc.relu(pats, dt)
        finite[0x8000] = False                                    # torch keeps -0; here -0 becomes +0
        assert np.array_equal(got[finite], want[finite])
        assert got[0x8000] == 0
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(10000).astype(np.float32),
                        np.array([0.0, -0.0, 1e-45, -1e-45, 3e38, -3e38], np.float32)])
    want = torch.relu(torch.from_numpy(x)).numpy() + np.float32(0.0)      # -0 + 0 = +0
    got = orc.relu(x, orc.F32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_relu_backward_matches_torch_threshold_backward():
    import torch
    rng = np.random.default_rng(9)
    for dt, tdt in ((orc.F32, torch.float32), (orc.F16, torch.float16), (orc.BF16, torch.bfloat16)):
        xh = torch.from_numpy(rng.standard_normal(20000).astype(np.float32)).to(tdt)
        xh[::7] = 0.0
        xh[3::11] = -0.0
        gy = torch.from_numpy(rng.standard_normal(20000).astype(np.float32)).to(tdt)
        want = torch.ops.aten.threshold_backward(gy.float(), xh.float(), 0.0).to(tdt)
        bits = lambda t: t.view(torch.int32 if dt == orc.F32 else torch.int16).numpy().view(
            np.uint32 if dt == orc.F32 else np.uint16)
        src = (lambda t: t.numpy()) if dt == orc.F32 else bits
        got = orc.relu_backward(src(xh), src(gy), dt)
        want_bits = bits(want + 0.0) if dt == orc.F32 else bits(want)
        got_bits = got.view(np.uint32) if dt == orc.F32 else got
        zero_neg = np.uint32(0x80000000) if dt == orc.F32 else np.uint16(0x8000)
        want_bits = np.where(want_bits == zero_neg, 0, want_bits)      # a dropped gradient is +0 here
        kept = src(gy) == zero_neg if dt != orc.F32 else bits(gy) == zero_neg
        want_bits = np.where(kept & (got_bits == zero_neg), zero_neg, want_bits)   # a kept -0 gradient stays -0
        assert np.array_equal(got_bits, want_bits)


def test_grad_weight_against_explicit_loops_and_fractions():
    # the definition written out with exact rational arithmetic on a tiny case, and with plain
    # Python loops on a slightly larger one
    from fractions import Fraction
    import torch
    rng = np.random.default_rng(2)
    m, k, n = 5, 4, 3
    xh = torch.from_numpy(rng.standard_normal((m, k)).astype(np.float32)).to(torch.bfloat16)
    gy = torch.from_numpy(rng.standard_normal((m, n)).astype(np.float32)).to(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    got = orc.grad_weight(bits(xh), bits(gy), m, k, n, orc.BF16)
    assert got.shape == (n, k) and got.dtype == np.float64
    for j in range(n):
        for c in range(k):
            exact = sum(Fraction(float(gy[i, j])) * Fraction(float(xh[i, c])) for i in range(m))
            assert abs(Fraction(float(got[j, c])) - exact) <= abs(exact) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 200)
    m, k, n = 17, 9, 6
    xh = rng.standard_normal((m, k)).astype(np.float32)
    gy = rng.standard_normal((m, n)).astype(np.float32)
    got = orc.grad_weight(xh, gy, m, k, n, orc.F32)
    for j in range(n):
        for c in range(k):
            want = 0.0
            for i in range(m):
                want += float(gy[i, j]) * float(xh[i, c])
            assert abs(got[j, c] - want) <= 1e-12 * (1 + abs(want))
    # transposed operand check: a matrix with one non-zero entry lands where the definition says
    xh = np.zeros((m, k), np.float32); gy = np.zeros((m, n), np.float32)
    xh[3, 7] = 2.0; gy[3, 4] = 5.0
    got = orc.grad_weight(xh, gy, m, k, n, orc.F32)
    assert got[4, 7] == 10.0 and np.count_nonzero(got) == 1


def test_linear_forward_against_exact_rationals_loops_and_a_single_entry():
    # y = x W^T: exact rational arithmetic on a tiny bfloat16 case (the result must be the bfloat16
    # value nearest to the exact sum whenever that sum is not within 2^-24 of a tie), plain Python
    # loops on small-integer inputs (every sum exact, so the result is the rounded exact value), and
    # one non-zero entry per operand to pin which index is which
    from fractions import Fraction
    import torch
    rng = np.random.default_rng(5)
    m, k, n = 4, 6, 3
    x = torch.from_numpy(rng.standard_normal((m, k)).astype(np.float32)).to(torch.bfloat16)
    w = torch.from_numpy(rng.standard_normal((n, k)).astype(np.float32)).to(torch.bfloat16)
    bits = lambda t: t.contiguous().view(torch.int16).numpy().view(np.uint16)
    got = orc.widen(orc.linear_forward(bits(x), bits(w), m, k, n, orc.BF16), orc.BF16).reshape(m, n)
    for i in range(m):
        for j in range(n):
            exact = sum(Fraction(float(x[i, c])) * Fraction(float(w[j, c])) for c in range(k))
            ulp = Fraction(2) ** (int(np.frexp(float(abs(exact)))[1]) - 8) if exact != 0 else Fraction(0)
            assert abs(Fraction(float(got[i, j])) - exact) <= ulp / 2 + abs(exact) * Fraction(1, 2 ** 23)
    m, k, n = 7, 40, 5
    xi = rng.integers(-3, 4, (m, k)).astype(np.float32)
    wi = rng.integers(-3, 4, (n, k)).astype(np.float32) / 4
    for dtype, tdt in ((orc.F16, torch.float16), (orc.BF16, torch.bfloat16)):
        got = orc.widen(orc.linear_forward(bits(torch.from_numpy(xi).to(tdt)), bits(torch.from_numpy(wi).to(tdt)),
                                           m, k, n, dtype), dtype).reshape(m, n)
        for i in range(m):
            for j in range(n):
                want = 0.0
                for c in range(k):
                    want += float(xi[i, c]) * float(wi[j, c])           # exact: multiples of 1/4 below 2^10
                assert got[i, j] == float(torch.tensor(want, dtype=torch.float64).to(tdt))
    xo = np.zeros((m, k), np.float32); wo = np.zeros((n, k), np.float32)
    xo[2, 11] = 3.0; wo[4, 11] = 0.5
    got = orc.linear_forward(xo, wo, m, k, n, orc.F32).reshape(m, n)
    assert got[2, 4] == 1.5 and np.count_nonzero(got) == 1
