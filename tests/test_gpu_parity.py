"""GPU parity: libdaf (through the C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

from daf_inputs import BF16, F16, F32, Workload, make_config, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import hip_harness
    assert torch.cuda.is_available(), "GPU tests need cuda:0"
    return hip_harness


def _workload(dtype, n, gs, bits, seed, scale=1.0, rng_seed=0):
    g = torch.Generator().manual_seed(rng_seed)
    x = (torch.randn(n, generator=g) * scale).to(torch_dtype(dtype))
    G = (n + gs - 1) // gs
    if bits == "mixed":
        b = np.random.default_rng(rng_seed).choice([1, 2, 4, 8], G).astype(np.uint8)
    else:
        b = np.array([bits], dtype=np.uint8)
    return Workload(f"dt{dtype}_n{n}_g{gs}_b{bits}", x, dtype, gs, b, seed)


# reduced instances of the five configurations: several tiles plus a tail that the tile
# kernel does not cover; the oracle finishes each in seconds
@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (2, 3 / 64), (3, 3 / 32), (4, 1 / 64), (5, 1 / 16)])
def test_reduced_configs_full_parity(H, cfg, scale):
    for w in make_config(cfg, scale):
        print("case", w.name, tuple(w.x.shape), flush=True)
        H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("gs", [32, 64, 96, 128, 256, 512, 1024, 2048, 4096, 8192])
@pytest.mark.parametrize("bits", [1, 2, 4, 8, "mixed"])
def test_group_size_matrix(H, dtype, gs, bits):
    # a few tiles worth of groups plus a ragged tail
    n = 4096 * 2 + gs * 3 + 17 + (4096 * 6 if gs >= 2048 else 0)
    w = _workload(dtype, n, gs, bits, seed=0xABCDEF0123456789 % (1 << 64), rng_seed=gs + 7 * dtype)
    print("case", w.name, flush=True)
    H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("n", [1, 5, 31, 32, 33, 255, 256, 4095, 4096, 4097, 12288])
def test_small_and_ragged_sizes(H, dtype, n):
    for gs, bits in ((32, 4), (128, 2), (256, "mixed")):
        w = _workload(dtype, n, gs, bits, seed=n, rng_seed=n)
        print("case", w.name, flush=True)
        H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
def test_degenerate_groups(H, dtype):
    """Constant groups, all-zero groups with mixed signs of zero, subnormal ranges, ranges so
    small that the reciprocal overflows, huge magnitudes."""
    gs = 128 if dtype == F32 else 64
    n = 4096 * 3
    g = torch.Generator().manual_seed(5)
    x = torch.randn(n, generator=g)
    x[0:gs] = 1.75
    x[gs:2 * gs] = 0.0
    x[gs:2 * gs:2] = -0.0
    x[2 * gs:3 * gs] = -3.0
    x[3 * gs] = 1e-30
    x[3 * gs + 1:4 * gs] = 0.0
    if dtype == F32:
        x[4 * gs:5 * gs] = torch.arange(gs) * 1.4e-45             # subnormal grid
        x[5 * gs:6 * gs] = torch.randn(gs, generator=g) * 1e-37   # reciprocal of range*512 overflows
        x[6 * gs:7 * gs] = torch.randn(gs, generator=g) * 1e37
        x[4096:4096 + gs] = torch.randn(gs, generator=g) * 3e-38  # a second tile with a tiny group
    elif dtype == F16:
        x[4 * gs:5 * gs] = torch.arange(gs) * 5.96e-8             # fp16 subnormals
        x[5 * gs:6 * gs] = torch.randn(gs, generator=g) * 1e4
    else:
        x[4 * gs:5 * gs] = torch.randn(gs, generator=g) * 1e-38
        x[5 * gs:6 * gs] = torch.randn(gs, generator=g) * 1e37   # max - min must stay finite
    x = x.to(torch_dtype(dtype))
    for bits in (1, 2, 8, "mixed"):
        G = n // gs
        b = (np.random.default_rng(1).choice([1, 2, 4, 8], G).astype(np.uint8) if bits == "mixed"
             else np.array([bits], np.uint8))
        w = Workload(f"degenerate_dt{dtype}_b{bits}", x, dtype, gs, b, 11)
        print("case", w.name, flush=True)
        H.assert_full_parity(w, H.run_hip(w))


# full-size configurations: every word, min, scale and dequantized element against the oracle
@pytest.mark.timeout(400)
@pytest.mark.parametrize("cfg", [2, 3, 5])
def test_full_size_configs_whole_tensor(H, cfg):
    (w,) = make_config(cfg)
    print("case", w.name, tuple(w.x.shape), flush=True)
    res = H.run_hip(w)
    print("ran; oracle on the whole tensor", flush=True)
    H.assert_whole_parity(w, res)


@pytest.mark.timeout(600)
def test_full_size_resnet18_step_whole_tensors(H):
    """All 17 saved activations of the batch-256 step through the list entry points, as bench.py
    times them: quantize in forward order in one call, dequantize in reverse order in one call
    with every packed result alive, then every tensor compared in full with the oracle."""
    import paper_2507_07149_amd as daf
    ws = make_config(4)
    assert len(ws) == 17 and sum(w.numel for w in ws) == 590_872_576
    dev = "cuda:0"
    state = []
    for w in ws:
        x = w.x.reshape(-1).to(dev)
        plan = daf.daf_plan(tuple(w.x.shape), w.group_size, int(w.bits[0]))
        words = torch.full((plan.packed_words,), -1, dtype=torch.int32, device=dev)
        mn = torch.full((plan.num_groups,), float("nan"), device=dev)
        sc = torch.full((plan.num_groups,), float("nan"), device=dev)
        xh = torch.full_like(x, float("nan"))
        state.append((plan, x, words, mn, sc, xh))
    daf.daf_quantize_pack_batch([(p, x, w.seed, words, mn, sc) for w, (p, x, words, mn, sc, xh) in zip(ws, state)])
    daf.daf_unpack_dequantize_batch([(p, words, mn, sc, xh, None) for (p, x, words, mn, sc, xh) in reversed(state)])
    torch.cuda.synchronize()
    for t in reversed(range(17)):
        plan, x, words, mn, sc, xh = state[t]
        print("tensor", t, tuple(ws[t].x.shape), flush=True)
        H.assert_whole_parity(ws[t], H.HipResult(plan, words, mn, sc, xh, None))
        state[t] = None
        del x, xh, words


@pytest.mark.timeout(400)
@pytest.mark.parametrize("dtype,gs,bits,n_tiles", [(BF16, 64, "mixed", 20000), (F32, 256, 2, 26000),
                                                   (F16, 128, "mixed", 19000)])
def test_many_tiles_full_parity(H, dtype, gs, bits, n_tiles):
    """Several times more tiles than the GPU holds waves at once, so that workgroups are
    dispatched in many rounds: whole-tensor comparison (77-107 M elements)."""
    n = n_tiles * 4096 + 5 * gs + 3
    w = _workload(dtype, n, gs, bits, seed=77, rng_seed=n_tiles)
    print("case", w.name, flush=True)
    H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.parametrize("dtype", [F32, F16, BF16])
@pytest.mark.parametrize("bits", [1, 2, 8, "mixed"])
@pytest.mark.parametrize("n,gs", [(4096 * 9 + 77, 8192), (4096 * 12, 4096 * 4), (4096 * 7 + 4095, 4096 * 3),
                                  (50_176, 50_176), (393_216, 393_216), (100_003, 100_032), (5000, 5024),
                                  (4096 * 5 + 1, 4096 * 5 + 32)])
def test_groups_longer_than_a_tile(H, dtype, bits, n, gs):
    """Group sizes above 4096 elements take the two-pass route (tile min/max, per-group reduce,
    quantize with the group's statistics), up to one group for the whole tensor (the paper's
    per-tensor statistics; 50,176 and 393,216 are the shapes of its reduction experiment)."""
    w = _workload(dtype, n, gs, bits, seed=gs, rng_seed=n % 1000)
    print("case", w.name, flush=True)
    H.assert_full_parity(w, H.run_hip(w))


@pytest.mark.timeout(300)
def test_per_tensor_quantization_of_the_resnet50_activation(H):
    (w0,) = make_config(2)
    n = w0.numel
    w = Workload("resnet50_per_tensor", w0.x, F32, n, np.array([2], np.uint8), 1)
    res = H.run_hip(w)
    H.assert_sampled_parity(w, res, n_samples=10)       # one group: this compares everything
    from oracle import daf_oracle as orc
    mm = orc.minmax(w0.x.reshape(-1).numpy(), F32)
    assert res.mn.cpu().numpy()[0] == mm[0]


@pytest.mark.timeout(900)
def test_more_than_two_to_the_32_elements(H):
    """Element indices beyond 32 bits: a bfloat16 tensor of 2^32 + 12,488 elements (8.6 GB), 2-bit
    groups of 64, quantized and dequantized in one call each.  The oracle runs group by group on
    sampled groups: the first and the last ones (the last group has 8 elements), the groups on
    both sides of element 2^31 and of element 2^32 (where a 32-bit index would wrap: the Philox
    counter, the tile index and the word offset all pass through there), and random ones.  The
    activation is generated on the device in pieces; the host holds only the sampled groups, in
    arrays whose untouched pages are never committed."""
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    from daf_inputs import to_numpy_bits
    dev = "cuda:0"
    n, gs, b, seed = (1 << 32) + 3 * 4096 + 200, 64, 2, 0x1234_5678_9ABC
    free, _ = torch.cuda.mem_get_info()
    if free < 24 << 30:
        pytest.skip("needs 24 GB of free device memory")
    x = torch.empty(n, dtype=torch.bfloat16, device=dev)
    gen = torch.Generator(device=dev).manual_seed(99)
    piece = 1 << 28
    for lo in range(0, n, piece):
        hi = min(n, lo + piece)
        x[lo:hi] = (torch.randn(hi - lo, device=dev, generator=gen) * 3).to(torch.bfloat16)
    plan = daf.daf_plan((n,), gs, b)
    G = plan.num_groups
    off, total = orc.plan(n, gs, np.array([b], np.uint8))
    assert G == (n + gs - 1) // gs == off.size and plan.packed_words == total
    words = torch.empty(total, dtype=torch.int32, device=dev)
    mn, sc = torch.empty(G, device=dev), torch.empty(G, device=dev)
    daf.daf_quantize_pack(plan, x, seed, words, mn, sc)
    xh = torch.empty_like(x)
    daf.daf_unpack_dequantize(plan, words, mn, sc, xh)
    torch.cuda.synchronize()

    rng = np.random.default_rng(5)
    near = lambda e: np.arange(e // gs - 40, e // gs + 40)
    picks = np.unique(np.concatenate([np.arange(70), np.arange(G - 70, G), near(1 << 31), near(1 << 32),
                                      near((1 << 32) + 4096), rng.integers(0, G, 300)]))
    xb = np.zeros(n, dtype=np.uint16)                      # lazily committed: only the sampled groups are written
    ow = np.zeros(total, dtype=np.uint32)
    omn, osc = np.zeros(G, dtype=np.float32), np.zeros(G, dtype=np.float32)
    oxh = np.zeros(n, dtype=np.uint16)
    bits1 = np.array([b], np.uint8)
    for g in picks:
        g = int(g)
        lo, hi = g * gs, min((g + 1) * gs, n)
        xb[lo:hi] = to_numpy_bits(x[lo:hi].cpu())
        orc.quantize_pack_range(xb, BF16, gs, bits1, off, seed, g, g + 1, ow, omn, osc)
        nw = ((hi - lo) * b + 31) // 32
        o0 = int(off[g])
        assert mn[g].item() == omn[g] and sc[g].item() == osc[g], f"min/scale of group {g}"
        assert np.array_equal(words[o0:o0 + nw].cpu().numpy().view(np.uint32), ow[o0:o0 + nw]), f"words of group {g}"
        orc.unpack_dequantize_range(ow, omn, osc, bits1, off, n, gs, g, g + 1, oxh, BF16)
        assert np.array_equal(to_numpy_bits(xh[lo:hi].cpu()), oxh[lo:hi]), f"dequantized values of group {g}"
    # a property over every element, on the device in pieces: min is the group minimum, |x - xhat| <= scale + rounding
    full = (n // gs) * gs
    for lo in range(0, full, piece):
        hi = min(full, lo + piece)
        xs = x[lo:hi].float().reshape(-1, gs)
        g0, g1 = lo // gs, hi // gs
        assert torch.equal(mn[g0:g1], xs.amin(dim=1) + 0.0)
        err = (xs - xh[lo:hi].float().reshape(-1, gs)).abs()
        bound = sc[g0:g1, None] * (1 + 2.0 ** -20) + (xs.abs() + sc[g0:g1, None]) * 2.0 ** -8
        assert bool((err <= bound).all())
    plan.destroy()


def test_seed_changes_codes_and_is_reproducible(H):
    w = _workload(F32, 4096 * 4, 256, 2, seed=1)
    a = H.u32(H.run_hip(w).words)
    b = H.u32(H.run_hip(w).words)
    w2 = Workload(w.name, w.x, w.dtype, w.group_size, w.bits, seed=2)
    c = H.u32(H.run_hip(w2).words)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    # high seed word is part of the key
    w3 = Workload(w.name, w.x, w.dtype, w.group_size, w.bits, seed=1 + (1 << 32))
    assert not np.array_equal(a, H.u32(H.run_hip(w3).words))
    H.assert_full_parity(w3, H.run_hip(w3))


def test_plan_scan_large_mixed(H):
    """Offsets of 5.6 M groups (the size of the LLM configuration) against the oracle's scan."""
    import paper_2507_07149_amd as daf
    from oracle import daf_oracle as orc
    G, gs = 5_636_096, 64
    bits = np.random.default_rng(3).choice([2, 4, 8], G).astype(np.uint8)
    n = G * gs - 13                                             # short last group
    plan = daf.daf_plan((n,), gs, torch.from_numpy(bits).cuda())
    off, total = orc.plan(n, gs, bits)
    assert plan.packed_words == total
    assert np.array_equal(plan.offsets().numpy().view(np.uint32), off)


def test_abi_errors_on_device(H):
    import paper_2507_07149_amd as daf
    dev = "cuda:0"
    bad_bits = torch.tensor([2, 4, 3, 8], dtype=torch.uint8, device=dev)
    with pytest.raises(daf.DafError) as e:
        daf.daf_plan((4 * 64,), 64, bad_bits)
    assert e.value.status == -1
    plan = daf.daf_plan((1024,), 64, 2)
    x = torch.zeros(1024 + 4, device=dev)
    words = torch.zeros(plan.packed_words, dtype=torch.int32, device=dev)
    mn = torch.zeros(plan.num_groups, device=dev)
    sc = torch.zeros(plan.num_groups, device=dev)
    with pytest.raises(daf.DafError) as e:                      # x not 16-byte aligned
        daf.daf_quantize_pack(plan, x[1:1025], 0, words, mn, sc)
    assert e.value.status == -1
    with pytest.raises(daf.DafError):                           # bits given for a uniform plan
        daf.daf_unpack_dequantize(plan, words, mn, sc, x[:1024],
                                  bits=torch.full((plan.num_groups,), 2, dtype=torch.uint8, device=dev))
    with pytest.raises(ValueError):                             # too few widths: caught by the binding
        daf.daf_unpack_dequantize(plan, words, mn, sc, x[:1024], bits=bad_bits)
    daf.daf_quantize_pack(plan, x[:1024], 0, words, mn, sc)     # and the good call still works
    torch.cuda.synchronize()
    assert int(words.abs().sum()) == 0


def test_runs_on_a_side_stream(H):
    import paper_2507_07149_amd as daf
    w = _workload(F16, 4096 * 6 + 64, 128, "mixed", seed=9)
    ref = H.run_hip(w)
    s = torch.cuda.Stream()
    x = w.x.cuda()
    words = torch.empty_like(ref.words)
    mn = torch.empty_like(ref.mn)
    sc = torch.empty_like(ref.scale)
    xh = torch.empty_like(x)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        daf.daf_quantize_pack(ref.plan, x, w.seed, words, mn, sc, stream=s)
        daf.daf_unpack_dequantize(ref.plan, words, mn, sc, xh, stream=s)
    s.synchronize()
    assert torch.equal(words, ref.words) and torch.equal(mn, ref.mn) and torch.equal(xh, ref.xhat)


def test_calls_can_be_captured_in_a_hip_graph(H):
    """daf_quantize_pack / daf_unpack_dequantize only enqueue kernels (no allocation, memset or
    synchronization), so a caller may capture them; every replay must equal the eager result,
    also after the input changed between replays."""
    import paper_2507_07149_amd as daf
    ws = [_workload(F32, 4096 * 40 + 300, 256, 2, seed=3), _workload(BF16, 4096 * 33 + 64, 64, "mixed", seed=4),
          _workload(F32, 4096 * 24, 4096 * 8, 4, seed=5)]
    state = []
    for w in ws:
        r = H.run_hip(w)                      # eager reference; also builds the plan
        x = w.x.reshape(-1).cuda()
        state.append((w, r, x, torch.empty_like(r.words), torch.empty_like(r.mn), torch.empty_like(r.scale),
                      torch.empty_like(x)))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for w, r, x, words, mn, sc, xh in state:
            daf.daf_quantize_pack(r.plan, x, w.seed, words, mn, sc)
            daf.daf_unpack_dequantize(r.plan, words, mn, sc, xh)
    for replay in range(3):
        if replay == 1:                        # new input values, same buffers
            for w, r, x, *_ in state:
                x.mul_(-1.5)
        graph.replay()
        torch.cuda.synchronize()
        for w, r, x, words, mn, sc, xh in state:
            if replay == 0:
                assert torch.equal(words, r.words) and torch.equal(mn, r.mn) and torch.equal(xh, r.xhat)
            else:
                w2 = Workload(w.name, x.cpu().reshape(w.x.shape), w.dtype, w.group_size, w.bits, w.seed)
                H.assert_full_parity(w2, H.HipResult(r.plan, words, mn, sc, xh, None))
