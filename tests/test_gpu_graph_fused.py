"""The fused and the list entry points only enqueue kernels (no allocation, no memset, no
synchronization), so a caller may capture them in a HIP graph.  Every replay must reproduce the
eager call bit for bit (all of these kernels add in a fixed order), also after the inputs
changed between replays; the program's own eager work runs between the replays."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_fused_and_list_calls_in_a_hip_graph():
    import paper_2507_07149_amd as daf
    dev = "cuda:0"
    g = torch.Generator().manual_seed(21)
    M, N, K, gs = 512, 512, 640, 64                    # 128-column tile, m in slices (workspace in use)
    G = M * K // gs
    bits = torch.from_numpy(np.random.default_rng(3).choice([1, 2, 4, 8], G).astype(np.uint8)).to(dev)
    plan = daf.daf_plan((M, K), gs, bits)
    plan_u = daf.daf_plan((M, K), gs, 4)
    z = torch.randn(M * K, generator=g).to(torch.bfloat16).to(dev)
    gy = (torch.randn(M, N, generator=g) * 0.3).to(torch.bfloat16).to(dev)
    gz_in = torch.randn(M * K, generator=g).to(torch.bfloat16).to(dev)

    def buffers(p):
        return (torch.empty(p.packed_words, dtype=torch.int32, device=dev), torch.empty(p.num_groups, device=dev),
                torch.empty(p.num_groups, device=dev))

    ws_bytes = daf.daf_unpack_matmul_workspace_bytes(plan, N, K)
    assert ws_bytes > 0

    def run(out):
        """All calls on the current stream, results into the tensors of `out`."""
        daf.daf_relu_quantize_pack(plan, z, 7, out["y"], *out["q"])
        daf.daf_unpack_relu_backward(plan, *out["q"], gz_in, out["gz"])
        daf.daf_unpack_matmul_grad_weight(plan, *out["q"], gy, out["dw"], out["ws"])
        daf.daf_quantize_pack_batch([(plan, out["y"], 9, *out["qb0"]), (plan_u, z, 10, *out["qb1"])])
        daf.daf_unpack_dequantize_batch([(plan, *out["qb0"], out["xh0"], None), (plan_u, *out["qb1"], out["xh1"], None)])

    def fresh():
        return dict(y=torch.empty_like(z), q=buffers(plan), gz=torch.empty_like(z), dw=torch.empty(N, K, device=dev),
                    ws=torch.empty(ws_bytes, dtype=torch.uint8, device=dev), qb0=buffers(plan), qb1=buffers(plan_u),
                    xh0=torch.empty_like(z), xh1=torch.empty_like(z))

    def same(a, b):
        for k in a:
            if k == "ws":
                continue
            xs, ys = (a[k], b[k]) if isinstance(a[k], tuple) else ((a[k],), (b[k],))
            for x, y in zip(xs, ys):
                assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), k

    captured = fresh()
    run(captured)                                       # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(captured)
    for replay in range(3):
        if replay == 1:                                 # new values in the same input buffers
            z.mul_(-0.75)
            gy.add_(0.125)
        for t in captured.values():                     # poison the outputs between replays
            for x in (t if isinstance(t, tuple) else (t,)):
                x.view(torch.uint8).fill_(0xA5)
        graph.replay()
        torch.cuda.synchronize()
        eager = fresh()
        run(eager)                                      # the program's own eager work between replays
        torch.cuda.synchronize()
        same(captured, eager)
    plan.destroy()
    plan_u.destroy()


def test_row_sized_and_long_groups_in_a_hip_graph():
    """The kernels for group sizes that are not a power of two (one wave per run of groups, one
    workgroup per long group, the workgroup-per-group tail) enqueue only kernels as well."""
    import paper_2507_07149_amd as daf
    dev = "cuda:0"
    g = torch.Generator().manual_seed(22)
    M, N, K = 512, 256, 640
    n = M * K + 1000                                   # a short last group for both plans
    G1 = (n + 639) // 640
    bits = torch.from_numpy(np.random.default_rng(4).choice([1, 2, 4, 8], G1).astype(np.uint8)).to(dev)
    plan_row = daf.daf_plan((n,), 640, bits)           # 20 units per group
    plan_long = daf.daf_plan((n,), 6400, 2)            # 200 units per group: two waves per group
    plan_mm = daf.daf_plan((M, K), 640, 4)             # one group per row, for the weight gradient
    plan_long.set_output_cached(True)
    z = torch.randn(n, generator=g).to(torch.float16).to(dev)
    gy = (torch.randn(M, N, generator=g) * 0.3).to(torch.float16).to(dev)

    def buffers(p):
        return (torch.empty(p.packed_words, dtype=torch.int32, device=dev), torch.empty(p.num_groups, device=dev),
                torch.empty(p.num_groups, device=dev))

    ws_bytes = daf.daf_unpack_matmul_workspace_bytes(plan_mm, N, K)

    def run(out):
        daf.daf_relu_quantize_pack(plan_row, z, 7, out["y"], *out["q0"])
        daf.daf_quantize_pack(plan_long, out["y"], 8, *out["q1"])
        daf.daf_quantize_pack_metrics(plan_row, z, 9, *out["q2"], out["met"])
        daf.daf_group_minmax(plan_row, z, out["lo"], out["hi"])
        daf.daf_quantize_pack_batch([(plan_row, z, 11, *out["q3"]), (plan_long, z, 12, *out["q4"])])
        daf.daf_unpack_dequantize(plan_long, *out["q1"], out["xh1"])
        daf.daf_unpack_dequantize_batch([(plan_row, *out["q3"], out["xh3"], None), (plan_long, *out["q4"], out["xh4"], None)])
        daf.daf_quantize_pack(plan_mm, z[: M * K], 13, *out["q5"])
        daf.daf_unpack_matmul_grad_weight(plan_mm, *out["q5"], gy, out["dw"], out["ws"])

    def fresh():
        return dict(y=torch.empty_like(z), q0=buffers(plan_row), q1=buffers(plan_long), q2=buffers(plan_row),
                    met=torch.empty(plan_row.num_groups, 3, device=dev), lo=torch.empty(plan_row.num_groups, device=dev),
                    hi=torch.empty(plan_row.num_groups, device=dev), q3=buffers(plan_row), q4=buffers(plan_long),
                    xh1=torch.empty_like(z), xh3=torch.empty_like(z), xh4=torch.empty_like(z), q5=buffers(plan_mm),
                    dw=torch.empty(N, K, device=dev, dtype=torch.float32),
                    ws=torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev))

    def same(a, b):
        for k in a:
            if k == "ws":
                continue
            xs, ys = (a[k], b[k]) if isinstance(a[k], tuple) else ((a[k],), (b[k],))
            for x, y in zip(xs, ys):
                assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), k

    captured = fresh()
    run(captured)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(captured)
    for replay in range(3):
        if replay == 1:
            z.mul_(-0.5)
            gy.add_(0.25)
        for t in captured.values():
            for x in (t if isinstance(t, tuple) else (t,)):
                x.view(torch.uint8).fill_(0xA5)
        graph.replay()
        torch.cuda.synchronize()
        eager = fresh()
        run(eager)
        torch.cuda.synchronize()
        same(captured, eager)
    for p in (plan_row, plan_long, plan_mm):
        p.destroy()
