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


def test_statistics_widths_plan_quantize_replayed_from_a_hip_graph():
    """The sequence a training loop runs every iteration (per-group statistics -> widths -> new
    offsets -> quantize) is captured once into a HIP graph and replayed on fresh activations:
    none of the four calls allocates, copies through the host, clears memory with a memset node or
    synchronizes.  Every replay is checked against the oracle, with the program's own eager work
    and synchronizations between the replays."""
    dtype, gs, classes = BF16, 64, (2, 4, 8)
    n = 4096 * 37 + 64 * 5
    G = (n + gs - 1) // gs
    dev = "cuda:0"
    gen = torch.Generator().manual_seed(123)
    x_dev = torch.zeros(n, dtype=torch_dtype(dtype), device=dev)
    stats_plan = daf.daf_plan((n,), gs, 8)
    plan = daf.daf_plan((n,), gs, torch.full((G,), 8, dtype=torch.uint8, device=dev))
    mn_s, mx_s = torch.empty(G, device=dev), torch.empty(G, device=dev)
    bits = torch.empty(G, dtype=torch.uint8, device=dev)
    ws = daf.daf_select_bits_workspace(G)
    words = torch.zeros(plan.packed_words_bound, dtype=torch.int32, device=dev)
    mn, sc = torch.empty(G, device=dev), torch.empty(G, device=dev)

    def sequence():
        daf.daf_group_minmax(stats_plan, x_dev, mn_s, mx_s)
        daf.daf_select_bits(mn_s, mx_s, classes, bits, ws)
        plan.update(bits)
        daf.daf_quantize_pack(plan, x_dev, 9, words, mn, sc)

    def check(x_cpu):
        xb = to_numpy_bits(x_cpu)
        gmin, gmax = orc.group_minmax(xb, dtype, gs)
        want_bits = orc.select_bits(gmin, gmax, classes)
        ow, omn, osc, _ = orc.quantize_pack(xb, dtype, gs, want_bits, 9)
        assert np.array_equal(bits.cpu().numpy(), want_bits)
        assert np.array_equal(words[: ow.size].cpu().numpy().view(np.uint32), ow)
        assert np.array_equal(mn.cpu().numpy().view(np.uint32), omn.view(np.uint32))
        assert np.array_equal(sc.cpu().numpy().view(np.uint32), osc.view(np.uint32))
        return ow.size

    side = torch.cuda.Stream()
    x0 = (torch.randn(n, generator=gen) * 3).to(torch_dtype(dtype))
    x_dev.copy_(x0)
    with torch.cuda.stream(side):                       # once eagerly on the capture stream
        side.wait_stream(torch.cuda.current_stream())
        sequence()
    torch.cuda.synchronize()
    check(x0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sequence()
    for trial in range(4):
        xt = (torch.randn(n, generator=gen) * (0.5 + trial)).to(torch_dtype(dtype))
        if trial == 2:
            xt[: n // 2] = 1.5                          # many equal ranges: ties across blocks
        x_dev.copy_(xt)
        words.fill_(-1)
        eager = torch.randn(1 << 16, device=dev).sum()  # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        total = check(xt)
        plan.finish()
        assert plan.packed_words == total
        assert torch.isfinite(eager)
    del graph
    plan.destroy()
    stats_plan.destroy()
