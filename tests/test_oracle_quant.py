"""Pins for the oracle's arithmetic: Eq. 1 closed forms, brute force in double precision,
error bound, unbiasedness over 4096 seeds, degenerate groups, Eq. 5 identity."""
import numpy as np
import pytest

from oracle import daf_oracle as orc

K = 8                                   # random bits per element (frozen)


def group_view(x, gs):
    n = x.size
    G = (n + gs - 1) // gs
    return [x[g * gs:min((g + 1) * gs, n)] for g in range(G)]


@pytest.mark.parametrize("b", [1, 2, 4, 8])
def test_min_scale_brute_force(b):
    rng = np.random.default_rng(b)
    n, gs = 500, 96
    x = (rng.standard_normal(n) * rng.choice([1e-3, 1.0, 1e4])).astype(np.float32)
    _, mn, sc, _ = orc.quantize_pack(x, orc.F32, gs, [b], 1)
    L = (1 << b) - 1
    for g, xs in enumerate(group_view(x, gs)):
        assert mn[g] == xs.min()
        rng64 = float(xs.max()) - float(xs.min())
        assert abs(float(sc[g]) * L - rng64) <= rng64 * 2.0 ** -22
        # scale is the correctly rounded quotient of the float32 range by L
        rng32 = np.float32(xs.max()) - np.float32(xs.min())
        assert sc[g] == np.float32(rng32) / np.float32(L)


@pytest.mark.parametrize("b", [1, 2, 4, 8])
@pytest.mark.parametrize("seed", [0, 1, 99])
def test_grid_points_reproduce_eq1_round(b, seed):
    """x = min + j*scale (Eq. 1's own grid) must quantize to j for every seed: on the grid
    the fractional part is ~0 so stochastic rounding is deterministic and equals `round`."""
    L = (1 << b) - 1
    mnv, mxv = np.float32(-0.7), np.float32(2.9)
    reps = 64 // (L + 1) if L < 63 else 1
    j = np.tile(np.arange(L + 1), max(reps, 1))[: max(64, L + 1)]
    if j.size % 32:
        j = np.concatenate([j, np.zeros(-j.size % 32, dtype=j.dtype)])
    j[0], j[1] = 0, L                                     # make sure both ends are present
    x = (np.float64(mnv) + j * (np.float64(mxv) - np.float64(mnv)) / L).astype(np.float32)
    x[0], x[1] = mnv, mxv
    _, mn, sc, codes = orc.quantize_pack(x, orc.F32, x.size, [b], seed, want_codes=True)
    assert mn[0] == mnv
    assert np.array_equal(codes, j.astype(np.uint8))
    # Eq. 1 evaluated in double with round-half-even (ties do not occur here)
    q = np.rint((x.astype(np.float64) - float(mnv)) / ((float(mxv) - float(mnv)) / L))
    assert np.array_equal(codes, q.astype(np.uint8))


@pytest.mark.parametrize("dtype", [orc.F32, orc.F16, orc.BF16])
@pytest.mark.parametrize("b", [1, 2, 4, 8])
def test_codes_bracket_double_precision_value_and_error_bound(dtype, b):
    rng = np.random.default_rng(17 + b)
    n, gs = 64 * 40, 64
    xf = (rng.standard_normal(n) * 2.5).astype(np.float32)
    x = xf if dtype == orc.F32 else orc.narrow(xf, dtype)
    xw = orc.widen(x, dtype).astype(np.float64)
    L = (1 << b) - 1
    words, mn, sc, codes = orc.quantize_pack(x, dtype, gs, [b], 3, want_codes=True)
    xh, _ = orc.unpack_dequantize(words, mn, sc, [b], n, gs, orc.F32)
    g = np.arange(n) // gs
    rngv = (sc.astype(np.float64) * L)[g]
    v = (xw - mn.astype(np.float64)[g]) * L / rngv                     # Eq. 1 argument, double
    lo = np.floor(v - 1e-4)
    hi = np.floor(v + 1e-4) + 1
    c = codes.astype(np.float64)
    assert np.all(c >= np.maximum(lo, 0)) and np.all(c <= np.minimum(hi, L))
    assert codes.max() <= L
    # |x - xhat| <= scale (plus float32 slack)
    err = np.abs(xw - xh.astype(np.float64))
    assert np.all(err <= sc.astype(np.float64)[g] * (1 + 2.0 ** -20) + rngv * 2.0 ** -22)
    # each group reaches code 0 at its min and code L at its max
    for gi in range(n // gs):
        s = slice(gi * gs, (gi + 1) * gs)
        assert codes[s][np.argmin(xw[s])] == 0
        assert codes[s][np.argmax(xw[s])] == L


def test_b1_codes_are_binary_and_scale_is_range():
    rng = np.random.default_rng(5)
    x = rng.standard_normal(256).astype(np.float32)
    _, mn, sc, codes = orc.quantize_pack(x, orc.F32, 128, [1], 2, want_codes=True)
    assert set(np.unique(codes)) <= {0, 1}
    for g, xs in enumerate(group_view(x, 128)):
        assert sc[g] == xs.max() - xs.min()


def test_unbiased_over_4096_seeds():
    """Mean of xhat over seeds 0..4095 converges to x: per element within 6 sigma of the
    Bernoulli mean plus the 2^-(k+1) granularity of P(up); the average signed deviation over
    all elements (in units of scale) is far below 1e-3.  A floor- or ceil-style compare
    instead of the midpoint compare shifts that average by 2^-9 ~ 2e-3 and fails."""
    rng = np.random.default_rng(2024)
    n, gs, b = 512, 128, 2
    x = rng.standard_normal(n).astype(np.float32)
    L = (1 << b) - 1
    S = 4096
    acc = np.zeros(n, dtype=np.float64)
    for seed in range(S):
        words, mn, sc, _ = orc.quantize_pack(x, orc.F32, gs, [b], seed)
        xh, _ = orc.unpack_dequantize(words, mn, sc, [b], n, gs, orc.F32)
        acc += xh
    mean = acc / S
    g = np.arange(n) // gs
    scale = sc.astype(np.float64)[g]
    v = (x.astype(np.float64) - mn.astype(np.float64)[g]) / scale
    f = v - np.floor(v)
    tol = 6 * scale * np.sqrt(f * (1 - f) / S) + scale * 2.0 ** -(K + 1) + scale * L * 2.0 ** -22
    dev = mean - x.astype(np.float64)
    assert np.all(np.abs(dev) <= tol)
    assert abs((dev / scale).mean()) < 1e-3
    # the empirical P(up) matches the fractional part (correlation check against a sign flip)
    p_up = (mean - (mn.astype(np.float64)[g] + np.floor(v) * scale)) / scale
    inner = (f > 0.05) & (f < 0.95)
    assert np.corrcoef(p_up[inner], f[inner])[0, 1] > 0.995


def test_probability_of_rounding_up_is_the_half_down_rounded_fraction():
    """Exhaustive over the 256 values of r for a few fractions: the number of r that round
    up must be ceil(f*256 - 1/2) (midpoint compare), counted through real oracle calls by
    placing the same x at 4096 consecutive element indices (16 per Philox block)."""
    b, gs = 2, 4096
    L = 3
    for frac in (0.0, 0.001, 0.25, 0.3, 0.5, 0.7071, 0.998, 0.9999):
        x = np.full(gs, 1.0 + frac, dtype=np.float32)
        x[0], x[1] = 0.0, 3.0                                # min 0, max 3 -> scale 1, v = x
        seed = 31
        _, mn, sc, codes = orc.quantize_pack(x, orc.F32, gs, [b], seed, want_codes=True)
        assert (mn[0], sc[0]) == (0.0, 1.0)
        f = float(x[2]) - 1.0                                 # exact fractional part in float32
        thresh = int(np.ceil(f * 256 - 0.5))
        r = np.array([orc.rand(seed, i) for i in range(2, gs)])
        want = 1 + (r < thresh).astype(np.uint8)
        assert np.array_equal(codes[2:], want), frac


def test_constant_group_and_tiny_range():
    x = np.full(64, 3.25, dtype=np.float32)
    x[32:] = np.float32(1e-42)                                # second group constant too (subnormal)
    words, mn, sc, codes = orc.quantize_pack(x, orc.F32, 32, [4], 0, want_codes=True)
    assert np.all(codes == 0) and np.all(words == 0)
    assert list(mn) == [np.float32(3.25), np.float32(1e-42)] and list(sc) == [0.0, 0.0]
    xh, _ = orc.unpack_dequantize(words, mn, sc, [4], 64, 32, orc.F32)
    assert np.array_equal(xh, x)
    # range so small that L/range overflows: codes are 0, scale is still range/L
    y = np.zeros(32, dtype=np.float32)
    y[5] = np.float32(2.0 ** -140)
    _, mn, sc, codes = orc.quantize_pack(y, orc.F32, 32, [8], 0, want_codes=True)
    assert np.all(codes == 0) and mn[0] == 0 and sc[0] == np.float32(2.0 ** -140) / np.float32(255)


def test_negative_zero_min_is_canonical():
    x = np.zeros(32, dtype=np.float32)
    x[::2] = -0.0
    _, mn, sc, _ = orc.quantize_pack(x, orc.F32, 32, [2], 0)
    assert mn.view(np.uint32)[0] == 0 and sc.view(np.uint32)[0] == 0
    x[3] = 1.0
    _, mn, sc, _ = orc.quantize_pack(x, orc.F32, 32, [2], 0)
    assert mn.view(np.uint32)[0] == 0


def test_code_clamped_at_top_level():
    """The group maximum must never produce code L+1, whatever the seed."""
    rng = np.random.default_rng(1)
    for trial in range(200):
        x = (rng.standard_normal(32) * 10 ** rng.uniform(-3, 3)).astype(np.float32)
        for b in (2, 8):
            _, _, _, codes = orc.quantize_pack(x, orc.F32, 32, [b], trial, want_codes=True)
            assert codes.max() == (1 << b) - 1


def test_eq5_bit_trick_matches_integer_to_float_conversion():
    """Eq. 5: the bit pattern 0x4B000000 | X read as float32 is 2^23 + X; subtracting 2^23
    gives float(X).  The oracle converts codes with an ordinary cast; both must agree for
    every 8-bit code (dequantize with min 0, scale 1)."""
    X = np.arange(256, dtype=np.uint32)
    trick = (X | np.uint32(0x4B000000)).view(np.float32) - np.float32(2.0 ** 23)
    words = X.astype(np.uint8).reshape(-1, 4)
    words = (words[:, 0].astype(np.uint32) << 24 | words[:, 1].astype(np.uint32) << 16
             | words[:, 2].astype(np.uint32) << 8 | words[:, 3].astype(np.uint32))
    xh, codes = orc.unpack_dequantize(words, np.zeros(1, np.float32), np.ones(1, np.float32), [8],
                                      256, 256, orc.F32, want_codes=True)
    assert np.array_equal(codes, X.astype(np.uint8))
    assert np.array_equal(xh, trick)


@pytest.mark.parametrize("dtype", [orc.F32, orc.F16, orc.BF16])
def test_dequantize_endpoints_and_double_recomputation(dtype):
    rng = np.random.default_rng(13)
    G, gs, b = 16, 32, 4
    L = 15
    mn = rng.standard_normal(G).astype(np.float32)
    sc = np.abs(rng.standard_normal(G)).astype(np.float32) / 7
    codes = rng.integers(0, L + 1, G * gs).astype(np.uint8)
    codes[::gs] = 0
    codes[1::gs] = L
    from tests.test_oracle_pack import bitstring_pack
    words = bitstring_pack(codes, G * gs, gs, [b])
    xh, back = orc.unpack_dequantize(words, mn, sc, [b], G * gs, gs, dtype, want_codes=True)
    assert np.array_equal(back, codes)
    xw = orc.widen(xh, dtype)
    g = np.arange(G * gs) // gs
    exact = codes.astype(np.float64) * sc.astype(np.float64)[g] + mn.astype(np.float64)[g]
    f32 = exact.astype(np.float32)                      # one rounding of the exact value = fmaf
    if dtype == orc.F32:
        assert np.array_equal(xw, f32)
        assert np.array_equal(xw[::gs], mn)             # code 0 gives min exactly
    else:
        assert np.array_equal(xh, orc.narrow(f32, dtype))


@pytest.mark.parametrize("dtype", [orc.F32, orc.F16, orc.BF16])
def test_whole_tensor_minmax_against_numpy(dtype):
    """Pins for the per-tensor reduction: numpy's min/max on the widened values, the position
    of the extremes anywhere in the array, single elements, and +0 for a zero result."""
    rng = np.random.default_rng(31 + dtype)
    for n in (1, 2, 63, 64, 65, 1000, 50_176, 393_216):
        xf = (rng.standard_normal(n) * 10 ** rng.uniform(-3, 3)).astype(np.float32)
        x = xf if dtype == orc.F32 else orc.narrow(xf, dtype)
        w = orc.widen(x, dtype)
        got = orc.minmax(x, dtype)
        assert got[0] == w.min() and got[1] == w.max()
        for pos in (0, n - 1, n // 2):                       # extremes at the ends and in the middle
            y = w.copy()
            y[pos] = w.max() * 2 + 1
            y[(pos + 1) % n if n > 1 else 0] = min(w.min() * 2 - 1, y[(pos + 1) % n if n > 1 else 0]) if n > 1 else y[0]
            yy = y if dtype == orc.F32 else orc.narrow(y, dtype)
            yw = orc.widen(yy, dtype)
            g = orc.minmax(yy, dtype)
            assert g[0] == yw.min() and g[1] == yw.max()
    z = np.zeros(8, dtype=np.float32)
    z[::2] = -0.0
    zz = z if dtype == orc.F32 else orc.narrow(z, dtype)
    g = orc.minmax(zz, dtype)
    assert g.view(np.uint32)[0] == 0 and g.view(np.uint32)[1] == 0
    neg = -np.abs(rng.standard_normal(100)).astype(np.float32) - 1
    nn = neg if dtype == orc.F32 else orc.narrow(neg, dtype)
    g = orc.minmax(nn, dtype)
    assert g[1] == orc.widen(nn, dtype).max() < 0


def test_one_group_is_per_tensor_quantization():
    """group_size >= N gives the paper's own granularity (Eq. 1 with tensor-wide min and max):
    min and scale must be those of the whole-tensor reduction."""
    rng = np.random.default_rng(77)
    n = 5000
    x = rng.standard_normal(n).astype(np.float32)
    gs = 5024                                                 # multiple of 32, >= n
    for b in (2, 4):
        _, mn, sc, codes = orc.quantize_pack(x, orc.F32, gs, [b], 5, want_codes=True)
        mm = orc.minmax(x, orc.F32)
        assert mn.size == 1 and mn[0] == mm[0]
        assert sc[0] == (mm[1] - mm[0]) / np.float32((1 << b) - 1)
        assert codes[np.argmin(x)] == 0 and codes[np.argmax(x)] == (1 << b) - 1
