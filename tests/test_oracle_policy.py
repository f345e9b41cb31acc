"""Pins for the oracle's per-group statistics and the rank-quantile width rule."""
import numpy as np
import pytest

from daf_inputs import bits_by_range_quantiles, make_config, to_numpy_bits
from oracle import daf_oracle as orc


@pytest.mark.parametrize("dtype", [orc.F32, orc.F16, orc.BF16])
@pytest.mark.parametrize("n,gs", [(64, 32), (1000, 96), (4096 + 5, 128), (777, 1024)])
def test_group_minmax_against_numpy(dtype, n, gs):
    rng = np.random.default_rng(n + gs)
    xf = (rng.standard_normal(n) * 3).astype(np.float32)
    x = xf if dtype == orc.F32 else orc.narrow(xf, dtype)
    w = orc.widen(x, dtype)
    mn, mx = orc.group_minmax(x, dtype, gs)
    G = (n + gs - 1) // gs
    assert mn.size == G
    for g in range(G):
        seg = w[g * gs:min((g + 1) * gs, n)]
        assert mn[g] == seg.min() and mx[g] == seg.max()
    # the quantizer's stored min is the same statistic
    _, qmn, qsc, _ = orc.quantize_pack(x, dtype, gs, [8], 0)
    assert np.array_equal(qmn.view(np.uint32), mn.view(np.uint32))


def test_group_minmax_zero_is_positive():
    x = np.zeros(64, dtype=np.float32)
    x[::3] = -0.0
    mn, mx = orc.group_minmax(x, orc.F32, 32)
    assert not mn.view(np.uint32).any() and not mx.view(np.uint32).any()


def lexsort_rule(gmin, gmax, classes):
    """The rule written with numpy's lexsort (an independent library sort)."""
    rng = gmax.astype(np.float32) - gmin.astype(np.float32)
    G = rng.size
    order = np.lexsort((np.arange(G), rng))
    rank = np.empty(G, dtype=np.int64)
    rank[order] = np.arange(G)
    return np.asarray(classes, np.uint8)[(rank * len(classes)) // G]


@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 7, 64, 1000, 4097, 100_003])
@pytest.mark.parametrize("classes", [(1, 2, 4, 8), (2, 4, 8), (4, 8), (2,)])
def test_select_bits_against_lexsort(G, classes):
    rng = np.random.default_rng(G)
    gmin = rng.standard_normal(G).astype(np.float32)
    gmax = gmin + np.abs(rng.standard_normal(G)).astype(np.float32)
    assert np.array_equal(orc.select_bits(gmin, gmax, classes), lexsort_rule(gmin, gmax, classes))


@pytest.mark.parametrize("classes", [(1, 2, 4, 8), (2, 4, 8)])
def test_select_bits_with_many_ties(classes):
    """Equal ranges are ordered by group index; constant (range 0) groups are the common case."""
    rng = np.random.default_rng(9)
    G = 10_007
    gmin = np.zeros(G, dtype=np.float32)
    gmax = rng.choice([0.0, 0.0, 0.0, 0.5, 1.0, 1.0, 2.0], G).astype(np.float32)
    got = orc.select_bits(gmin, gmax, classes)
    assert np.array_equal(got, lexsort_rule(gmin, gmax, classes))
    # class sizes are the equal-count split whatever the ties
    C = len(classes)
    want_counts = np.bincount((np.arange(G) * C) // G, minlength=C)
    assert np.array_equal(np.array([(got == c).sum() for c in classes]), want_counts)
    # all-equal keys: classes follow the group index
    same = orc.select_bits(np.zeros(G, np.float32), np.ones(G, np.float32), classes)
    assert np.array_equal(same, np.asarray(classes, np.uint8)[(np.arange(G) * C) // G])


def test_select_bits_reproduces_the_benchmark_workloads():
    """The generators' own width assignment (numpy) equals the oracle's rule on the oracle's
    per-group statistics."""
    for cfg, scale, classes in ((3, 1 / 16, (1, 2, 4, 8)), (5, 1 / 16, (2, 4, 8))):
        (w,) = make_config(cfg, scale)
        mn, mx = orc.group_minmax(to_numpy_bits(w.x), w.dtype, w.group_size)
        assert np.array_equal(orc.select_bits(mn, mx, classes), w.bits)


@pytest.mark.parametrize("dtype", [orc.F32, orc.F16, orc.BF16])
def test_group_metrics_against_numpy(dtype):
    """Quantization error and magnitude per group, recomputed with numpy from the quantizer's
    codes: xhat is the single rounding to binary32 of code*scale+min evaluated exactly."""
    rng = np.random.default_rng(40 + dtype)
    n, gs = 128 * 9 + 50, 128
    G = (n + gs - 1) // gs
    bits = rng.choice([1, 2, 4, 8], G).astype(np.uint8)
    xf = (rng.standard_normal(n) * 2).astype(np.float32)
    x = xf if dtype == orc.F32 else orc.narrow(xf, dtype)
    w = orc.widen(x, dtype).astype(np.float64)
    words, mn, sc, codes = orc.quantize_pack(x, dtype, gs, bits, 6, want_codes=True)
    got = orc.group_metrics(x, dtype, gs, codes, mn, sc)
    g = np.arange(n) // gs
    xhat = (codes.astype(np.float64) * sc.astype(np.float64)[g] + mn.astype(np.float64)[g]).astype(np.float32)
    err = np.bincount(g, weights=(w - xhat.astype(np.float64)) ** 2, minlength=G)
    mag = np.bincount(g, weights=w ** 2, minlength=G)
    assert np.allclose(got[:, 0], err, rtol=1e-12, atol=0) and np.allclose(got[:, 1], mag, rtol=1e-12, atol=0)
    if dtype == orc.F32:        # for binary32 tensors xhat is exactly what dequantize returns
        xh, _ = orc.unpack_dequantize(words, mn, sc, bits, n, gs, orc.F32)
        assert np.array_equal(xh, xhat)
    # more bits, less error; error bounded by n_g * scale^2
    lens = np.minimum(gs, n - gs * np.arange(G))
    assert np.all(got[:, 0] <= lens * sc.astype(np.float64) ** 2 * (1 + 1e-6) + 1e-30)


def test_group_variance_closed_form_and_sampling():
    """Quantization variance per group: (1) against the closed form in numpy (the number of
    random bytes that round an element up is ceil(256 f - 1/2) clipped to [0, 256], f the
    fractional part of the binary32 product), (2) against the sample variance of the dequantized
    values over many seeds of the oracle's own quantizer."""
    rng = np.random.default_rng(77)
    n, gs = 64 * 6, 64
    G = n // gs
    bits = np.array([1, 2, 4, 8, 2, 4], np.uint8)
    x = (rng.standard_normal(n) * 3).astype(np.float32)
    got = orc.group_variance(x, orc.F32, gs, bits)
    g = np.arange(n) // gs
    mn, mx = orc.group_minmax(x, orc.F32, gs)
    L = (2.0 ** bits.astype(np.float64) - 1).astype(np.float32)
    rng_ = (mx - mn).astype(np.float32)
    scale = (rng_ / L).astype(np.float32)
    inv = (L / rng_).astype(np.float32)
    v = ((x - mn[g]).astype(np.float32) * inv[g]).astype(np.float32)
    f = (v - np.floor(v)).astype(np.float64)
    T = np.clip(np.ceil(256.0 * f - 0.5), 0, 256)
    p = T / 256.0
    want = np.bincount(g, weights=p * (1 - p), minlength=G) * scale.astype(np.float64) ** 2
    assert np.allclose(got, want, rtol=1e-12, atol=0)
    # sampling: the variance of xhat over seeds, summed per group
    seeds = 3000
    acc = np.zeros((seeds, n), np.float64)
    for s in range(seeds):
        _, omn, osc, codes = orc.quantize_pack(x, orc.F32, gs, bits, 1000 + s, want_codes=True)
        acc[s] = codes.astype(np.float64) * osc.astype(np.float64)[g] + omn.astype(np.float64)[g]
    sample = np.bincount(g, weights=acc.var(axis=0), minlength=G)
    assert np.all(np.abs(sample - got) <= 0.08 * got + 1e-12), (sample, got)
    # a constant group has no variance; neither has a group whose values sit on the levels
    assert orc.group_variance(np.full(64, 2.5, np.float32), orc.F32, 64, 4)[0] == 0.0
    lv = np.tile(np.arange(4, dtype=np.float32), 16)
    assert orc.group_variance(lv, orc.F32, 64, 2)[0] == 0.0
