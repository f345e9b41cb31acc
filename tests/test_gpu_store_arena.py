"""The paged activation store driving the GPU path: the store decides widths and page offsets
under a memory budget, daf_quantize_pack writes words, min and scale straight into the arena
at those offsets, daf_unpack_dequantize reads them back, and everything equals the oracle at
the widths the store chose (Sec. 3.4 feeding Sec. 2.2 / 3.3)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _sizes(n, gs, widths):
    G = -(-n // gs)
    return [4 * G * (-(-gs * w // 32)) + 8 * G for w in widths]


def test_store_places_quantized_activations_in_one_arena():
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    from paper_2507_07149_amd import store

    dev = torch.device("cuda:0")
    gen = torch.Generator().manual_seed(77)
    shapes = [(8, 64, 32, 32), (4, 197, 768), (8, 128, 16, 16), (2, 512, 1024), (16, 32, 28, 28), (4, 64, 56, 56)]
    gs, widths, page = 256, [8, 4, 2, 1], 4096
    xs = [torch.relu(torch.randn(s, generator=gen)) for s in shapes]
    importance = [3.0, 9.0, 0.5, 6.0, 1.5, 4.0]
    sizes = [_sizes(x.numel(), gs, widths) for x in xs]
    budget = int(0.45 * sum(s[0] for s in sizes))          # forces narrower widths and an eviction or two
    st = store.Store(page, budget, None, 64 * page)
    for i, (x, s) in enumerate(zip(xs, sizes)):
        st.add(i, widths, s, [1000 + x.numel() // 1000] * 4, importance[i])
    decisions = [st.receive(i, importance[i] * f) for i, f in enumerate((1.0, 1.2, 0.8, 0.3, 2.0, 1.0))]
    assert st.validate() and st.used_bytes() <= budget
    assert any(d[0] == 0 for d in decisions) or any(0 < d[0] < 8 for d in decisions)
    arena = torch.zeros(st.capacity_bytes() // 4, dtype=torch.int32, device=dev)

    kept = []
    for i, (x, (bits, off, size)) in enumerate(zip(xs, decisions)):
        if bits == 0:
            continue
        plan = daf.daf_plan(tuple(x.shape), gs, bits)
        G, W = plan.num_groups, plan.packed_words
        assert size == 4 * W + 8 * G and off % page == 0 and off + size <= st.capacity_bytes()
        base = off // 4
        words = arena[base: base + W]
        mn = arena[base + W: base + W + G].view(torch.float32)
        sc = arena[base + W + G: base + W + 2 * G].view(torch.float32)
        daf.daf_quantize_pack(plan, x.reshape(-1).to(dev), 500 + i, words, mn, sc)
        kept.append((i, x, bits, plan, words, mn, sc))
    torch.cuda.synchronize()

    for i, x, bits, plan, words, mn, sc in reversed(kept):          # backward order
        xh = torch.empty(x.numel(), device=dev)
        daf.daf_unpack_dequantize(plan, words, mn, sc, xh)
        torch.cuda.synchronize()
        ow, omn, osc, _ = orc.quantize_pack(x.numpy().reshape(-1), daf.F32, gs, bits, 500 + i)
        oxh, _ = orc.unpack_dequantize(ow, omn, osc, bits, x.numel(), gs, daf.F32)
        assert np.array_equal(words.cpu().numpy().view(np.uint32), ow), f"activation {i}: words differ"
        assert np.array_equal(mn.cpu().numpy().view(np.uint32), omn.view(np.uint32))
        assert np.array_equal(sc.cpu().numpy().view(np.uint32), osc.view(np.uint32))
        assert np.array_equal(xh.cpu().numpy().view(np.uint32), oxh.view(np.uint32)), f"activation {i}: xhat differs"
        st.release(i)
        plan.destroy()
    assert st.used_bytes() == 0 and st.validate()
