"""GPU parity of the several-tensors-per-call entry points: every tensor of a list must come
out exactly as the oracle (and therefore the single-tensor calls) produce it, whatever mix of
plans the list holds (shared launches, separate launches, remainders after the last tile)."""
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


def _roundtrip(daf, orc, dtype, specs):
    """specs: list of (n, gs, bits) with bits an int or 'mixed'."""
    g = torch.Generator().manual_seed(123 + dtype)
    tensors, q_items, d_items, keep = [], [], [], []
    for i, (n, gs, bits) in enumerate(specs):
        x = (torch.randn(n, generator=g) * (1 + i)).to(torch_dtype(dtype))
        G = (n + gs - 1) // gs
        b = (np.random.default_rng(i).choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed"
             else np.array([bits], np.uint8))
        dbits = torch.from_numpy(b).cuda() if b.size > 1 else None
        plan = daf.daf_plan((n,), gs, dbits if dbits is not None else int(b[0]))
        xd = x.cuda()
        words = torch.full((max(plan.packed_words, 1),), -1, dtype=torch.int32, device="cuda:0")[: plan.packed_words]
        mn = torch.full((G,), float("nan"), device="cuda:0")
        sc = torch.full((G,), float("nan"), device="cuda:0")
        xh = torch.zeros_like(xd)
        tensors.append((x, gs, b, 40 + i, words, mn, sc, xh))
        q_items.append((plan, xd, 40 + i, words, mn, sc))
        d_items.append((plan, words, mn, sc, xh, None))
        keep.append((plan, xd, dbits))
    print("case", dtype, specs, flush=True)
    daf.daf_quantize_pack_batch(q_items)
    daf.daf_unpack_dequantize_batch(d_items)
    torch.cuda.synchronize()
    for i, (x, gs, b, seed, words, mn, sc, xh) in enumerate(tensors):
        ow, omn, osc, _ = orc.quantize_pack(to_numpy_bits(x), dtype, gs, b, seed)
        oxh, _ = orc.unpack_dequantize(ow, omn, osc, b, x.numel(), gs, dtype)
        assert np.array_equal(words.cpu().numpy().view(np.uint32), ow), f"tensor {i}: words differ"
        assert np.array_equal(mn.cpu().numpy().view(np.uint32), omn.view(np.uint32)), f"tensor {i}: min differs"
        assert np.array_equal(sc.cpu().numpy().view(np.uint32), osc.view(np.uint32)), f"tensor {i}: scale differs"
        assert np.array_equal(to_numpy_bits(xh.cpu()).view(oxh.dtype), oxh), f"tensor {i}: xhat differs"
    for plan, _, _ in keep:
        plan.destroy()


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
def test_batch_of_like_tensors_shares_launches(env, dtype):
    daf, orc = env
    _roundtrip(daf, orc, dtype, [(4096 * 3, 256, 2), (4096 * 7, 256, 2), (4096, 256, 2), (4096 * 2 + 256 * 3 + 40, 256, 2)])


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
def test_batch_of_unlike_tensors(env, dtype):
    daf, orc = env
    _roundtrip(daf, orc, dtype, [(4096 * 2, 128, 4), (4096 * 2, 128, 8), (4096 * 3, 64, "mixed"), (4096 * 5 + 64, 64, "mixed"),
                                 (1000, 96, 2), (20000, 8192, 1), (4096 * 2, 128, 4), (33, 32, "mixed")])


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
def test_batch_of_tensors_with_row_sized_groups(env, dtype):
    """Group sizes that are not a power of two share one launch whatever their size, as long as
    the width kind is the same; power-of-two items in between keep their own batches."""
    daf, orc = env
    _roundtrip(daf, orc, dtype, [(768 * 40, 768, 2), (3072 * 9 + 5, 3072, 2), (96 * 100 + 96 * 3, 96, 2), (4096 * 3, 256, 2),
                                 (160 * 77 + 33, 160, 2), (768 * 11, 768, "mixed"), (4064 * 3 + 1500, 4064, "mixed"),
                                 (4096 * 2, 64, "mixed"), (2080 * 7, 2080, 8), (11008 * 3 + 100, 11008, 8)])


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_batch_of_tensors_with_long_groups(env, dtype):
    """Groups of 4128 ... 65536 elements: items with the same number of waves per group and the same
    width kind share a launch; others, and the short last groups, get their own."""
    daf, orc = env
    _roundtrip(daf, orc, dtype, [(11008 * 5, 11008, 2), (11008 * 3 + 700, 11008, 2), (12288 * 2 + 5, 12288, 2), (4128 * 7, 4128, 2),
                                 (8192 * 300, 8192, 2), (4096 * 3, 256, 2), (11008 * 4, 11008, "mixed"), (9600 * 6 + 9000, 9600, "mixed"),
                                 (32736 * 2 + 1, 32736, 8), (768 * 9, 768, 8), (32768 * 3, 32768, 8), (65504 * 2 + 9, 65504, 8),
                                 (40000 * 3, 40000, 2)])


def test_batch_of_many_row_sized_tensors(env):
    daf, orc = env
    _roundtrip(daf, orc, BF16, [(768 * (5 + i % 4), 768 if i % 3 else 3072, 4) for i in range(40)])


def test_batch_longer_than_one_launch(env):
    daf, orc = env
    _roundtrip(daf, orc, F32, [(4096 * (1 + i % 3), 256, 2) for i in range(70)])


@pytest.mark.timeout(400)
def test_batch_resnet18_step_at_full_size(env):
    """The 17 tensors of the ResNet-18 configuration at full size, one call per direction;
    compared with the single-tensor calls (which the full-size parity tests tie to the oracle)."""
    daf, _ = env
    ws = make_config(4, 1.0)
    q_items, d_items, ref = [], [], []
    for w in ws:
        x = w.x.reshape(-1).cuda()
        plan = daf.daf_plan(tuple(w.x.shape), w.group_size, int(w.bits[0]))
        bufs = [torch.empty(plan.packed_words, dtype=torch.int32, device="cuda:0"),
                torch.empty(plan.num_groups, device="cuda:0"), torch.empty(plan.num_groups, device="cuda:0")]
        xh = torch.empty_like(x)
        q_items.append((plan, x, w.seed, *bufs))
        d_items.append((plan, *bufs, xh, None))
        ref.append((plan, x, w.seed, bufs, xh))
    print("case resnet18 step, 17 tensors", flush=True)
    daf.daf_quantize_pack_batch(q_items)
    daf.daf_unpack_dequantize_batch(d_items)
    torch.cuda.synchronize()
    for plan, x, seed, bufs, xh in ref:
        w2, m2, s2 = torch.empty_like(bufs[0]), torch.empty_like(bufs[1]), torch.empty_like(bufs[2])
        daf.daf_quantize_pack(plan, x, seed, w2, m2, s2)
        xh2 = torch.empty_like(xh)
        daf.daf_unpack_dequantize(plan, w2, m2, s2, xh2)
        torch.cuda.synchronize()
        assert torch.equal(w2, bufs[0]) and torch.equal(m2.view(torch.int32), bufs[1].view(torch.int32))
        assert torch.equal(s2.view(torch.int32), bufs[2].view(torch.int32))
        assert torch.equal(xh2.view(torch.int32), xh.view(torch.int32))
        plan.destroy()


def test_batch_argument_errors(env):
    daf, _ = env
    plan = daf.daf_plan((4096,), 256, 2)
    x = torch.zeros(4096 + 1, device="cuda:0")
    words = torch.zeros(plan.packed_words, dtype=torch.int32, device="cuda:0")
    mn = torch.zeros(plan.num_groups, device="cuda:0")
    with pytest.raises(daf.DafError) as e:                       # second item misaligned: nothing is launched
        daf.daf_quantize_pack_batch([(plan, x[:4096], 0, words, mn, mn), (plan, x[1:], 0, words, mn, mn)])
    assert e.value.status == -1
    lib = daf.load_library()
    assert lib.daf_quantize_pack_batch(None, 1, 0, None) == -1
    assert lib.daf_unpack_dequantize_batch(None, 0, 0, None) == -1
