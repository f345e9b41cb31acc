"""daf_quantize_pack_static (the entry point that allocates nothing: the two-pass route keeps
its per-tile and per-group statistics in a static device buffer of the library) against
daf_quantize_pack, bit for bit, through the C ABI; two calls in a row on the shared buffer, the
second with a smaller input, so that stale contents of the first would show."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2507_07149_amd as daf
from daf_inputs import BF16, F16, F32, torch_dtype

pytestmark = pytest.mark.gpu


def _run(entry, plan, x, seed):
    dev = x.device
    words = torch.full((plan.packed_words,), -1, dtype=torch.int32, device=dev)
    mn = torch.full((plan.num_groups,), float("nan"), device=dev)
    sc = torch.full((plan.num_groups,), float("nan"), device=dev)
    entry(plan, x, seed, words, mn, sc)
    torch.cuda.synchronize()
    return words, mn, sc


def _case(dtype, n, gs, bits, seed):
    g = torch.Generator().manual_seed(n % 9973 + gs)
    x = (torch.randn(n, generator=g) * 3).to(torch_dtype(dtype)).cuda()
    G = (n + gs - 1) // gs
    if bits == "mixed":
        b = torch.from_numpy(np.random.default_rng(gs).choice([1, 2, 4, 8], G).astype(np.uint8)).cuda()
    else:
        b = bits
    plan = daf.daf_plan((n,), gs, b)
    print("case dtype", dtype, "n", n, "gs", gs, "bits", bits, "route", plan.quantize_route(x.dtype), flush=True)
    ref = _run(daf.daf_quantize_pack, plan, x, seed)
    got = _run(daf.daf_quantize_pack_static, plan, x, seed)
    for name, r, g_ in zip(("words", "min", "scale"), ref, got):
        assert torch.equal(r.view(torch.int32), g_.view(torch.int32)), f"{name} differ"
    return plan


def test_static_scratch_equals_plan_scratch_two_calls_in_a_row():
    # one group for the whole tensor (the paper's per-tensor statistics): two-pass route
    n1 = 4096 * 3001 + 77
    p1 = _case(F32, n1, ((n1 + 31) // 32) * 32, 2, seed=5)
    assert p1.quantize_route(torch.float32) == "two_pass"
    # right after it, a smaller tensor with other values and another dtype on the same buffer
    n2 = 4096 * 37 + 5
    p2 = _case(BF16, n2, ((n2 + 31) // 32) * 32, 4, seed=6)
    assert p2.quantize_route(torch.bfloat16) == "two_pass"
    # several long groups, per-group widths; and the first size again after the small one
    _case(F16, 131072 * 9, 131072, "mixed", seed=7)
    _case(F32, n1, ((n1 + 31) // 32) * 32, 2, seed=8)


def test_plans_without_scratch_go_through_unchanged():
    for dtype, n, gs, bits in ((F32, 4096 * 50 + 300, 256, 2), (BF16, 4096 * 20, 64, "mixed"), (F16, 768 * 100, 768, 8)):
        _case(dtype, n, gs, bits, seed=n)


def test_oversized_plan_is_refused_before_any_launch():
    n = (1 << 31) - 32                                       # 524288 tiles: 4 MiB of pairs, limit 2 MiB
    plan = daf.daf_plan((n,), n, 1)
    L = daf.load_library()
    small = torch.zeros(64, device="cuda:0")
    rc = L.daf_quantize_pack_static(plan.handle, small.data_ptr(), 0, 0, small.data_ptr(), small.data_ptr(),
                                    small.data_ptr(), None)
    assert rc == -5 and b"scratch" in L.daf_status_string(rc)
    assert daf.STATIC_SCRATCH_BYTES == 2 << 20
    # just inside the limit: 8 * (tiles + 1) <= 2 MiB
    ok = daf.daf_plan(((262143 * 4096),), 262143 * 4096, 1)
    assert 8 * (262143 + 1) <= daf.STATIC_SCRATCH_BYTES
    ok.destroy()
    plan.destroy()
