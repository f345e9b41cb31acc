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
