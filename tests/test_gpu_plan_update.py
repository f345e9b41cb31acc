"""daf_plan_update: widths change on the stream with no host round trip (statistics -> widths ->
plan -> quantize); the packed output equals the oracle's for the new widths."""
import numpy as np
import pytest
import torch

import paper_2507_07149_amd as daf
from daf_inputs import BF16, F16, F32, Workload, make_config, to_numpy_bits, torch_dtype
from oracle import daf_oracle as orc

pytestmark = pytest.mark.gpu


def _quantize_and_compare(plan, x_cpu, dtype, gs, bits_np, seed):
    dev = "cuda:0"
    x = x_cpu.to(dev)
    G = plan.num_groups
    words = torch.full((plan.packed_words,), -1, dtype=torch.int32, device=dev)       # the bound, or exact
    mn = torch.empty(G, device=dev)
    sc = torch.empty(G, device=dev)
    xh = torch.empty_like(x)
    daf.daf_quantize_pack(plan, x, seed, words, mn, sc)
    daf.daf_unpack_dequantize(plan, words, mn, sc, xh)
    torch.cuda.synchronize()
    ow, omn, osc, _ = orc.quantize_pack(to_numpy_bits(x_cpu), dtype, gs, bits_np, seed)
    oxh, _ = orc.unpack_dequantize(ow, omn, osc, bits_np, x_cpu.numel(), gs, dtype)
    assert np.array_equal(words[: ow.size].cpu().numpy().view(np.uint32), ow)
    assert np.array_equal(mn.cpu().numpy().view(np.uint32), omn.view(np.uint32))
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), osc.view(np.uint32))
    assert np.array_equal(to_numpy_bits(xh.cpu()), oxh)
    return ow.size


@pytest.mark.parametrize("dtype,gs,n", [(F32, 256, 4096 * 9 + 300), (BF16, 64, 4096 * 30 + 64 * 3 + 5), (F16, 128, 4096 * 12)])
def test_update_then_quantize_without_sync(dtype, gs, n):
    g = torch.Generator().manual_seed(n)
    x = (torch.randn(n, generator=g) * 2).to(torch_dtype(dtype))
    G = (n + gs - 1) // gs
    rng = np.random.default_rng(gs)
    bits_a = rng.choice([1, 2, 4, 8], G).astype(np.uint8)
    bits_b = rng.choice([2, 4, 8], G).astype(np.uint8)
    d_a, d_b = torch.from_numpy(bits_a).cuda(), torch.from_numpy(bits_b).cuda()
    plan = daf.daf_plan((n,), gs, d_a)
    exact_a = plan.packed_words
    assert _quantize_and_compare(plan, x, dtype, gs, bits_a, 3) == exact_a
    plan.update(d_b)                                      # enqueued only
    assert plan.packed_words == plan.packed_words_bound >= exact_a
    total_b = _quantize_and_compare(plan, x, dtype, gs, bits_b, 4)
    plan.finish()
    assert plan.packed_words == total_b
    off, total = orc.plan(n, gs, bits_b)
    assert total == total_b and np.array_equal(plan.offsets().numpy().view(np.uint32), off)
    plan.update(d_a)                                      # and back
    plan.finish()
    assert plan.packed_words == exact_a
    plan.destroy()


def test_invalid_width_in_an_update_is_made_safe_and_reported():
    n, gs = 4096 * 4, 128
    G = n // gs
    x = torch.randn(n, generator=torch.Generator().manual_seed(1))
    good = np.full(G, 2, np.uint8)
    bad = good.copy()
    bad[5] = 3
    bad[77] = 0
    plan = daf.daf_plan((n,), gs, torch.from_numpy(good).cuda())
    plan.update(torch.from_numpy(bad).cuda())
    fixed = bad.copy()
    fixed[[5, 77]] = 8                                    # what the plan's copy holds
    _quantize_and_compare(plan, x, F32, gs, fixed, 9)
    with pytest.raises(daf.DafError) as e:
        plan.finish()
    assert e.value.status == -1
    plan.update(torch.from_numpy(good).cuda())
    plan.finish()
    plan.destroy()


def test_statistics_widths_plan_quantize_on_the_device():
    """The whole controller-side sequence on one stream for a reduced LLM-like tensor; widths and
    packed output equal the host-side rule + oracle."""
    (w,) = make_config(5, 1 / 16)
    dev = "cuda:0"
    x = w.x.reshape(-1).to(dev)
    G = w.num_groups
    plan = daf.daf_plan(tuple(w.x.shape), w.group_size, torch.full((G,), 8, dtype=torch.uint8, device=dev))
    lo, hi = torch.empty(G, device=dev), torch.empty(G, device=dev)
    bits = torch.empty(G, dtype=torch.uint8, device=dev)
    ws = daf.daf_select_bits_workspace(G)
    words = torch.empty(plan.packed_words_bound, dtype=torch.int32, device=dev)
    mn, sc = torch.empty(G, device=dev), torch.empty(G, device=dev)
    daf.daf_group_minmax(plan, x, lo, hi)
    daf.daf_select_bits(lo, hi, (2, 4, 8), bits, ws)
    plan.update(bits)
    daf.daf_quantize_pack(plan, x, w.seed, words, mn, sc)
    torch.cuda.synchronize()
    assert np.array_equal(bits.cpu().numpy(), w.bits)
    ow, omn, osc, _ = orc.quantize_pack(to_numpy_bits(w.x), w.dtype, w.group_size, w.bits, w.seed)
    assert np.array_equal(words[: ow.size].cpu().numpy().view(np.uint32), ow)
    assert np.array_equal(mn.cpu().numpy().view(np.uint32), omn.view(np.uint32))
    plan.finish()
    assert plan.packed_words == ow.size
    plan.destroy()
