"""Pins for the oracle's packing side: a text bit-string packer written from the layout
rule, the worked examples of Algorithm 2, closed-form sizes, and pack->unpack identity."""
import numpy as np
import pytest

from oracle import daf_oracle as orc


def bitstring_pack(codes, n, gs, bits):
    """Reference packer on text: per group, concatenate each code's b-bit binary form in
    element order, right-pad with '0' to a multiple of 32, cut into 32-character chunks."""
    G = (n + gs - 1) // gs
    words = []
    for g in range(G):
        b = int(bits[0] if len(bits) == 1 else bits[g])
        s = "".join(format(int(c), f"0{b}b") for c in codes[g * gs:min((g + 1) * gs, n)])
        s += "0" * (-len(s) % 32)
        words += [int(s[k:k + 32], 2) for k in range(0, len(s), 32)]
    return np.array(words, dtype=np.uint32)


def read_examples(golden_dir):
    out = []
    with open(f"{golden_dir}/alg2_unpack_examples.txt") as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            t = line.split()
            out.append((int(t[0]), int(t[1], 16), [int(v) for v in t[2:]]))
    return out


def test_algorithm2_worked_examples(golden_dir):
    """Unpack: the oracle must return the hand-written codes for the hand-written words.
    Dequantizing with min = 0, scale = 1 turns a code into the float of the same value."""
    ex = read_examples(golden_dir)
    assert len(ex) >= 6
    for b, word, codes in ex:
        n = 32 // b
        gs = 32
        words = np.array([word], dtype=np.uint32)
        xh, got = orc.unpack_dequantize(words, np.zeros(1, np.float32), np.ones(1, np.float32),
                                        [b], n, gs, orc.F32, want_codes=True)
        assert list(got) == codes, (b, hex(word))
        assert list(xh) == [float(c) for c in codes]
        # and the rule as printed for 4 bits: (w << 4j) >> 28
        if b == 4:
            assert [((word << (4 * j)) & 0xFFFFFFFF) >> 28 for j in range(8)] == codes


def _quantize_codes_are(x, gs, bits, seed=0):
    words, mn, sc, codes = orc.quantize_pack(x, orc.F32, gs, bits, seed, want_codes=True)
    return words, mn, sc, codes


@pytest.mark.parametrize("b", [1, 2, 4, 8])
@pytest.mark.parametrize("n,gs", [(32, 32), (64, 32), (100, 32), (513, 128), (96 * 5 + 7, 96)])
def test_pack_matches_bitstring_uniform(b, n, gs):
    rng = np.random.default_rng(100 * b + n)
    x = rng.standard_normal(n).astype(np.float32)
    words, mn, sc, codes = _quantize_codes_are(x, gs, [b], seed=5)
    assert codes.max() <= (1 << b) - 1
    want = bitstring_pack(codes, n, gs, [b])
    assert words.dtype == np.uint32 and np.array_equal(words, want)


def test_pack_matches_bitstring_mixed_and_offsets():
    rng = np.random.default_rng(3)
    n, gs = 64 * 37 + 11, 64
    G = (n + gs - 1) // gs
    bits = rng.choice([1, 2, 4, 8], G).astype(np.uint8)
    x = rng.standard_normal(n).astype(np.float32)
    words, mn, sc, codes = _quantize_codes_are(x, gs, bits, seed=9)
    assert np.array_equal(words, bitstring_pack(codes, n, gs, bits))
    off, total = orc.plan(n, gs, bits)
    lens = np.minimum(gs, n - gs * np.arange(G))
    w = (lens * bits.astype(np.int64) + 31) // 32
    assert total == w.sum() == words.size
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(w)[:-1]]).astype(np.uint32))


def test_b8_words_are_big_endian_bytes():
    rng = np.random.default_rng(8)
    x = rng.standard_normal(256).astype(np.float32)
    words, _, _, codes = _quantize_codes_are(x, 64, [8])
    assert np.array_equal(words.astype(">u4").view(np.uint8), codes)


def test_plan_closed_form_sizes(golden_dir):
    """Sizes of the five benchmark configurations (uniform ones through the oracle's plan;
    the mixed ones through class counts of the equal-count split)."""
    rows = {}
    with open(f"{golden_dir}/plan_sizes.txt") as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            c, n, gs, G, tot = [int(v) for v in line.split()]
            rows[c] = (n, gs, G, tot)
    for cfg, b in ((1, 2), (2, 2)):
        n, gs, G, tot = rows[cfg]
        off, total = orc.plan(n, gs, [b])
        assert (off.size, total) == (G, tot)
        assert off[-1] == tot - gs * b // 32
    # config 4 is 17 tensors; every N is a multiple of 256, so the sum is N*2/32
    n, gs, G, tot = rows[4]
    shapes = [(1, 64, 112), (4, 64, 56), (4, 128, 28), (4, 256, 14), (4, 512, 7)]
    acc_n = acc_w = 0
    for cnt, c, hw in shapes:
        nn = 256 * c * hw * hw
        _, t = orc.plan(nn, gs, [2])
        acc_n += cnt * nn
        acc_w += cnt * t
    assert (acc_n, acc_w) == (n, tot)
    # mixed configurations: equal-count classes, class k gets ranks with floor(rank*C/G) == k
    for cfg, classes in ((3, (1, 2, 4, 8)), (5, (2, 4, 8))):
        n, gs, G, tot = rows[cfg]
        rank = np.arange(G, dtype=np.int64)
        bits = np.asarray(classes, np.uint8)[(rank * len(classes)) // G]
        _, total = orc.plan(n, gs, bits)
        assert total == tot


def test_plan_rejects_bad_arguments():
    for bad in ([0], [3], [5], [16]):
        with pytest.raises(ValueError):
            orc.plan(64, 32, bad)
    with pytest.raises(ValueError):
        orc.plan(64, 48, [2])            # group size must be a multiple of 32
    with pytest.raises(ValueError):
        orc.plan(64, 32, [2, 2, 2])      # neither 1 nor G entries


@pytest.mark.parametrize("dtype", [orc.F32, orc.F16, orc.BF16])
def test_pack_unpack_identity_on_codes(dtype):
    rng = np.random.default_rng(21)
    n, gs = 128 * 19 + 40, 128
    G = (n + gs - 1) // gs
    bits = rng.choice([1, 2, 4, 8], G).astype(np.uint8)
    xf = (rng.standard_normal(n) * 3).astype(np.float32)
    x = xf if dtype == orc.F32 else orc.narrow(xf, dtype)
    words, mn, sc, codes = orc.quantize_pack(x, dtype, gs, bits, 77, want_codes=True)
    _, back = orc.unpack_dequantize(words, mn, sc, bits, n, gs, dtype, want_codes=True)
    assert np.array_equal(codes, back)


def test_short_last_group_pads_with_zero_bits():
    x = np.linspace(-1, 1, 32 + 5).astype(np.float32)
    words, _, _, codes = orc.quantize_pack(x, orc.F32, 32, [4], 0, want_codes=True)
    assert words.size == 4 + 1
    tail = int(words[-1])
    assert tail & ((1 << 12) - 1) == 0            # 5 codes * 4 bits used, 12 pad bits are zero
    assert [(tail >> (28 - 4 * j)) & 15 for j in range(5)] == list(codes[32:])
