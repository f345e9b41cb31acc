#!/usr/bin/env python3
"""Benchmark of the DAF activation quantize/pack hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--no-cpu-baseline]

A step is one pass of the whole hot path over one activation batch: daf_quantize_pack
(min/max, scale, stochastic-rounding quantize, pack) followed by daf_unpack_dequantize, with
all inputs resident in HBM.  Without --config the workload is the largest configuration, the 17
activations a ResNet-18 training step saves at batch 256 (fp32, 590.9 M elements, groups of
256, 2 bits; quantized in forward order by one list call, dequantized in reverse order by
another), and the line also carries `per_config`: kernel time, algorithmic bytes and roofline
fraction of both directions for the ResNet-50-like conv activation (configuration 2), the
ViT/BERT-like fp16 activation (3) and the LLM MLP bf16 activation (5).  Workloads smaller than
the 256 MB last-level cache rotate over several buffer sets, so loads come from HBM.

Prints ONE JSON line.  `value` is GB/s of activation bytes through the path: each step moves
the activation tensor once through quantize+pack and once through unpack+dequantize, so
value = 2 * N * sizeof(dtype) / step time.  Per-direction rates and the roofline of the
dominant kernel (algorithmic bytes / HIP-event kernel time, against 8 TB/s) ride along, as
does the CPU oracle timed on this host (a reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
# HBM bytes per launch (quantize+pack, unpack+dequantize) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this program, each scaled by what the same counter reads for a 1 GiB device copy; QUOTED from the named
# summary, not measured in the run that prints them (the JSON says so next to the figure).
QUOTED_TRAFFIC = {
    2: (220055818, 220159672, "profiles/quantize_dequantize_resnet50_conv_f32_64x256x56x56_g256_b2.md"),
    3: (65503175, 64721348, "profiles/quantize_dequantize_vit_bert_f16_32x1024x768_g128_b1248.md"),
    4: (2529705172, 2530220191, "profiles/quantize_dequantize_resnet18_step_f32_bs256_g256_b2.md"),
    5: (1000922059, 1002183800, "profiles/quantize_dequantize_llm_mlp_bf16_16x2048x11008_g64_b248.md"),
}
ROTATE_BYTES = 768 << 20          # buffer sets rotate over at least this much input
ROTATE_PACKED_BYTES = 512 << 20   # ... and over at least this much packed output (words, min, scale)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=None, choices=[1, 2, 3, 4, 5],
                    help="one configuration only; without it the headline is configuration 4 (the largest) and "
                         "configurations 2, 3 and 5 ride along as per_config records")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--minmax", action="store_true",
                    help="time daf_minmax (whole-tensor reduction, both methods) on the paper's two shapes "
                         "and on the default activation instead of the quantize/dequantize step")
    ap.add_argument("--device-widths", action="store_true",
                    help="for a per-group-width configuration (3 or 5): time the device-side sequence "
                         "daf_group_minmax -> daf_select_bits -> daf_plan that produces the widths and offsets")
    ap.add_argument("--group-size", type=int, default=None,
                    help="override the group size of a uniform-width configuration; 0 = one group per "
                         "tensor (the paper's per-tensor statistics)")
    ap.add_argument("--streams", type=int, default=1,
                    help="the timed steps launch independent tensors / independent batches round-robin on "
                         "this many HIP streams (default priority); with 2 the tail of one kernel overlaps "
                         "the start of the next; the per-kernel roofline timing always uses one stream")
    ap.add_argument("--fused-matmul", action="store_true",
                    help="time daf_unpack_matmul_grad_weight (unpack+dequantize inside the weight-gradient "
                         "product) against daf_unpack_dequantize followed by the library matrix product; "
                         "--config 5 (LLM MLP, bf16), 3 (ViT MLP, fp16) or 2 (conv activation as [N*H*W, C], fp32)")
    ap.add_argument("--fused-linear", action="store_true",
                    help="time daf_linear_quantize_pack (y = x W^T with the quantize+pack of y in the product's "
                         "epilogue) against the library matrix product followed by daf_quantize_pack; "
                         "--config 5 (LLM MLP up-projection, bf16, K = 4096) or 3 (ViT MLP down-projection, fp16, K = 3072: "
                         "the configuration's shape read as [M, 768] with groups of 128)")
    ap.add_argument("--f32", action="store_true",
                    help="with --fused-matmul: the same shape with binary32 tensors (32x32x2 MFMA, 157.3 TFLOP/s peak)")
    ap.add_argument("--uniform-bits", type=int, default=None, choices=[1, 2, 4, 8],
                    help="with --fused-matmul: one width for every group instead of the configuration's per-group widths")
    ap.add_argument("--fused-relu", action="store_true",
                    help="time daf_relu_quantize_pack (activation function fused into the quantize pass) "
                         "against a separate relu kernel followed by daf_quantize_pack")
    ap.add_argument("--output-policy", action="store_true",
                    help="time daf_unpack_dequantize alone and followed by a kernel that reads its output "
                         "(daf_group_minmax), with streaming and with cached output stores "
                         "(daf_plan_set_output_cached)")
    ap.add_argument("--sweep", action="store_true",
                    help="kernel-time map over element formats, group sizes (--sweep-group-sizes) and widths on one "
                         "tensor of 2^27 normal random elements: one line of JSON per case, fraction of 8 TB/s on "
                         "algorithmic bytes for quantize+pack and unpack+dequantize")
    ap.add_argument("--sweep-group-sizes", type=str, default="32,64,96,256,768,3072,4096,11008,16384",
                    help="comma-separated group sizes for --sweep")
    ap.add_argument("--list-rows", action="store_true",
                    help="16 fp16 tensors with per-group widths and one group per row: one quantize call per tensor "
                         "against one list call, for three tensor shapes")
    ap.add_argument("--page-store", action="store_true",
                    help="time the host-side paged activation store (red-black trees against re-sorting, and the "
                         "plain model) on synthetic iterations; uses no GPU")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a device copy of 1 GiB (a kernel of known traffic) so that the HBM "
                         "byte counters of a rocprofv3 --pmc run can be scaled against it")
    return ap.parse_args()


def algorithmic_bytes(w, total_words):
    """Bytes the method must move for one direction of one tensor: the activation once, the
    packed words once, min and scale once, plus (per-group widths only) one width byte per
    group and one 4-byte offset per group."""
    n, G = w.numel, w.num_groups
    esz = w.x.element_size()
    meta = 0 if w.bits.size == 1 else G * (1 + 4)
    return n * esz + 4 * total_words + 8 * G + meta


def bench_page_store(args, np):
    """One iteration = reset, pre-iteration estimation of all activations, then all of them
    arriving in the forward pass with importances that differ from the moving averages
    (Algorithm 3).  Budget = 35 % of the bytes at the widest width, so the reduction loop runs
    for most arrivals.  Reported: microseconds per iteration for the red-black-tree indices,
    for re-sorting at every selection, and for the plain Python model."""
    from oracle.page_store_oracle import PageStoreOracle
    from paper_2507_07149_amd import store
    page, widths = 64 << 10, [8, 4, 2, 1]
    rows = []
    for n in (64, 512, 4096):
        rng = np.random.default_rng(100 + n)
        numel = (rng.integers(1, 64, n) * 65536).astype(np.int64)               # elements per activation
        by = np.stack([numel * w // 8 + 8 * (numel // 256) for w in widths], 1)    # words + min/scale, group 256
        tm = np.stack([numel // 4000 + 2000 for _ in widths], 1).astype(np.int64)  # ~4 elements per ns + launch
        ma = rng.uniform(0.1, 10.0, n)
        imp = ma * rng.uniform(0.3, 3.0, n)
        ids = np.arange(n, dtype=np.int64)
        budget = int(by[:, 0].sum() * 0.35)
        res = {}
        for name, kind in (("rbtree", store.INDEX_RBTREE), ("sort", store.INDEX_SORT)):
            st = store.Store(page, budget, None, 100 << 20, index_kind=kind)
            reps = max(3, min(args.steps, 200000 // n))
            best = float("inf")
            for _ in range(reps):
                t = time.perf_counter()
                st.reset()
                st.add_many(ids, widths, by, tm, ma)
                bits, _, _ = st.receive_many(ids, imp)
                best = min(best, time.perf_counter() - t)
            res[name] = {"us_per_iteration": round(best * 1e6, 1), "selections": st.num_selections() // reps,
                         "stored": int((bits > 0).sum())}
            st.destroy()
        if n <= 512:
            o = PageStoreOracle(page, budget, None, 100 << 20)
            t = time.perf_counter()
            for i in range(n):
                o.add(int(ids[i]), widths, by[i].tolist(), tm[i].tolist(), float(ma[i]))
            ob = [o.receive(int(ids[i]), float(imp[i]))[0] for i in range(n)]
            res["python_model_us"] = round((time.perf_counter() - t) * 1e6, 1)
            assert ob == bits.tolist(), "the store and the model disagree"
        res["speedup_rbtree_over_sort"] = round(res["sort"]["us_per_iteration"] / res["rbtree"]["us_per_iteration"], 2)
        rows.append({"activations": n, **res})
    print(json.dumps({"metric": "paged activation store, microseconds per iteration of Algorithm 3",
                      "unit": "us", "higher_is_better": False, "data": "synthetic", "n_gpus": 0,
                      "config": {"workload": "page_store_budget35pct_page64KiB"}, "results": rows}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2507_07149_amd as daf
    from daf_inputs import CONFIG_NAMES, make_config, to_numpy_bits

    if args.page_store:
        bench_page_store(args, np)
        return
    if args.config is None and args.fused_linear:
        args.config = 5
    if args.config is None and (args.device_widths or args.fused_matmul or args.output_policy or args.fused_relu):
        args.config = 2

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    daf.load_library()                      # fails loudly if libdaf.so is missing
    dev = torch.device("cuda:0")

    import numpy as np
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4,
                                               "launches": args.steps}}))
        return

    if args.minmax:
        ws = daf.daf_minmax_workspace()
        out = torch.empty(2, device=dev)
        res = []
        shapes = [("conv2d_in_1x256x14x14", (1, 256, 14, 14)), ("attention_in_1x512x768", (1, 512, 768)),
                  ("resnet50_conv_64x256x56x56", (64, 256, 56, 56))]
        for name, shape in shapes:
            n = int(np.prod(shape))
            n_sets = max(1, min(64, -(-ROTATE_BYTES // (4 * n))))
            xs = [torch.randn(n, device=dev) for _ in range(n_sets)]
            row = {"shape": name, "elements": n, "dtype": "f32", "buffer_sets": n_sets}
            for label, method in (("two_pass", daf.REDUCE_TWO_PASS), ("atomic", daf.REDUCE_ATOMIC)):
                for i in range(args.warmup):
                    daf.daf_minmax(xs[i % n_sets], method, ws, out)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                reps = max(args.steps, 2 * n_sets)
                torch.cuda.synchronize()
                e0.record()
                for i in range(reps):
                    daf.daf_minmax(xs[i % n_sets], method, ws, out)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / reps
                row[label + "_us"] = round(us, 2)
                row[label + "_GBps"] = round(4 * n / us / 1e3, 1)
            res.append(row)
        print(json.dumps({"metric": "whole-tensor min/max reduction time per call", "unit": "us", "n_gpus": 1,
                          "data": "synthetic", "results": res}))
        return

    if args.device_widths:
        (w,) = make_config(args.config)
        classes = {3: (1, 2, 4, 8), 5: (2, 4, 8)}[args.config]
        x = w.x.reshape(-1).to(dev)
        stats_plan = daf.daf_plan(tuple(w.x.shape), w.group_size, 8)
        G = stats_plan.num_groups
        mn, mx = torch.empty(G, device=dev), torch.empty(G, device=dev)
        bits = torch.empty(G, dtype=torch.uint8, device=dev)
        ws = daf.daf_select_bits_workspace(G)

        def timed(fn, reps):
            for _ in range(args.warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps

        t_stats = timed(lambda: daf.daf_group_minmax(stats_plan, x, mn, mx), args.steps)
        t_select = timed(lambda: daf.daf_select_bits(mn, mx, classes, bits, ws), args.steps)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(10):
            daf.daf_plan(tuple(w.x.shape), w.group_size, bits).destroy()
        t_plan = (time.perf_counter() - t) * 1e6 / 10
        ok = bool((bits.cpu().numpy() == w.bits).all())
        # the same without a host round trip: one plan kept across iterations, its widths replaced
        # on the stream (daf_plan_update), the quantize launch right behind it
        plan = daf.daf_plan(tuple(w.x.shape), w.group_size, bits)
        words = torch.empty(plan.packed_words_bound, dtype=torch.int32, device=dev)
        qmn, qsc = torch.empty(G, device=dev), torch.empty(G, device=dev)
        t_update = timed(lambda: plan.update(bits), args.steps)

        def controller():
            daf.daf_group_minmax(stats_plan, x, mn, mx)
            daf.daf_select_bits(mn, mx, classes, bits, ws)
            plan.update(bits)

        def iteration():
            controller()
            daf.daf_quantize_pack(plan, x, w.seed, words, qmn, qsc)
        t_ctrl = timed(controller, args.steps)
        t_iter = timed(iteration, args.steps)

        # ... and with no pass over the activation for the widths at all: the next iteration's widths
        # come from the scales (and widths) the quantize call of this iteration left behind
        bits_next = bits.clone()

        def lagged_controller():
            daf.daf_select_bits_from_scale(qsc, bits_next, classes, bits_next, ws)
            plan.update(bits_next)

        def lagged_iteration():
            daf.daf_quantize_pack(plan, x, w.seed, words, qmn, qsc)
            lagged_controller()
        iteration()
        t_lag_ctrl = timed(lagged_controller, args.steps)
        t_lag_iter = timed(lagged_iteration, args.steps)
        plan.update(bits)
        # the same iteration captured once into a HIP graph and replayed (no call in it allocates,
        # synchronizes or copies through the host)
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            side.wait_stream(torch.cuda.current_stream())
            iteration()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            iteration()
        t_graph = timed(graph.replay, args.steps)
        bits_graph_ok = bool((bits.cpu().numpy() == w.bits).all())
        plan.finish()
        stats_bytes = w.numel * w.x.element_size() + 8 * G
        print(json.dumps({"metric": "device-side width selection", "unit": "us", "n_gpus": 1, "data": "synthetic",
                          "config": {"workload": CONFIG_NAMES[args.config], "groups": G},
                          "group_minmax_us": round(t_stats, 2),
                          "group_minmax_GBps": round(stats_bytes / t_stats / 1e3, 1),
                          "group_minmax_frac_of_8TBps": round(stats_bytes / t_stats / 1e3 / HBM_PEAK_GBPS, 4),
                          "select_bits_us": round(t_select, 2), "plan_us_with_sync": round(t_plan, 1),
                          "plan_update_us_no_sync": round(t_update, 2),
                          "widths_from_previous_scales_plan_us_no_sync": round(t_lag_ctrl, 2),
                          "quantize_then_widths_from_its_scales_plan_us_no_sync": round(t_lag_iter, 2),
                          "statistics_widths_plan_quantize_us_graph_replay": round(t_graph, 2),
                          "widths_match_generator_after_graph_replay": bits_graph_ok,
                          "statistics_widths_plan_us_no_sync": round(t_ctrl, 2),
                          "statistics_widths_plan_quantize_us_no_sync": round(t_iter, 2),
                          "packed_words_after_finish": plan.packed_words,
                          "widths_match_generator": ok}))
        return

    if args.fused_linear:
        (w,) = make_config(args.config)
        # The configuration's tensor is the OUTPUT y [M, N] of the layer (its shape, group size and
        # per-group widths); x and W are normal random operands scaled so that y has unit variance.
        N = w.x.shape[-1]
        M = w.numel // N
        K = {5: 4096, 3: 3072}.get(args.config, 1024)
        dt = w.x.dtype
        g = torch.Generator(device=dev).manual_seed(w.seed)
        x = torch.randn(M, K, device=dev, generator=g).to(dt)
        W = (torch.randn(N, K, device=dev, generator=g) / K ** 0.5).to(dt)
        bits = int(w.bits[0]) if w.bits.size == 1 else torch.from_numpy(w.bits).to(dev)
        if args.uniform_bits:
            bits = args.uniform_bits
        plan = daf.daf_plan((M, N), w.group_size, bits)
        G = plan.num_groups
        n_sets = 3
        outs = [(torch.empty(M, N, dtype=dt, device=dev), torch.empty(plan.packed_words, dtype=torch.int32, device=dev),
                 torch.empty(G, device=dev), torch.empty(G, device=dev)) for _ in range(n_sets)]
        it = [0]

        def timed(fn, reps):
            for _ in range(max(2, args.warmup // 4)):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        def fused():
            y, words, mn, sc = outs[it[0] % n_sets]
            it[0] += 1
            daf.daf_linear_quantize_pack(plan, x, W, w.seed, y, words, mn, sc)

        def library_mm():
            torch.mm(x, W.t(), out=outs[it[0] % n_sets][0])

        def unfused():
            y, words, mn, sc = outs[it[0] % n_sets]
            it[0] += 1
            torch.mm(x, W.t(), out=y)
            daf.daf_quantize_pack(plan, y.view(-1), w.seed, words, mn, sc)

        def product_only():
            daf.daf_linear_quantize_pack(plan, x, W, w.seed, outs[it[0] % n_sets][0], None, None, None)

        def own_mm_then_quantize():
            y, words, mn, sc = outs[it[0] % n_sets]
            it[0] += 1
            daf.daf_linear_quantize_pack(plan, x, W, w.seed, y, None, None, None)
            daf.daf_quantize_pack(plan, y.view(-1), w.seed, words, mn, sc)

        reps = max(3, min(args.steps, 20))
        t_fused = timed(fused, reps)
        t_unfused = timed(unfused, reps)
        t_mm = timed(library_mm, reps)
        t_own = timed(product_only, reps)
        t_own_unfused = timed(own_mm_then_quantize, reps)
        # the two products differ in the order of their binary32 additions: compare y, and the packed
        # output of the fused call with daf_quantize_pack applied to the y it wrote
        fused()
        yf, wf, mnf, scf = outs[(it[0] - 1) % n_sets]
        y_lib = torch.mm(x, W.t())
        rel = ((yf.float() - y_lib.float()).abs().max() / y_lib.float().abs().max()).item()
        w2, mn2, sc2 = torch.empty_like(wf), torch.empty_like(mnf), torch.empty_like(scf)
        daf.daf_quantize_pack(plan, yf.view(-1), w.seed, w2, mn2, sc2)
        torch.cuda.synchronize()
        same = bool(torch.equal(wf, w2) and torch.equal(mnf, mn2) and torch.equal(scf, sc2))
        flops = 2.0 * M * N * K
        ach = flops / (t_fused * 1e-3) / 1e12
        print(json.dumps({"metric": "linear layer forward with quantize+pack in the epilogue, TFLOP/s", "value": round(ach, 1),
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": reps, "data": "synthetic", "higher_is_better": True,
                          "dtype": {0: "f32", 1: "f16", 2: "bf16"}[w.dtype],
                          "config": {"workload": CONFIG_NAMES[args.config] + f"_linear_forward_K{K}", "M": M, "N": N, "K": K,
                                     "buffer_sets": n_sets},
                          "fused_ms": round(t_fused, 4), "library_mm_then_quantize_ms": round(t_unfused, 4),
                          "library_mm_alone_ms": round(t_mm, 4),
                          "library_mm_TFLOPs": round(flops / (t_mm * 1e-3) / 1e12, 1),
                          "same_kernel_without_quantization_ms": round(t_own, 4),
                          "same_kernel_without_quantization_then_quantize_ms": round(t_own_unfused, 4),
                          "epilogue_cost_ms": round(t_fused - t_own, 4),
                          "separate_quantize_pass_ms": round(t_own_unfused - t_own, 4),
                          "y_bytes_not_read_back": M * N * x.element_size(),
                          "max_rel_diff_of_y_vs_library": round(rel, 5),
                          "packed_output_equals_quantize_pack_of_own_y": same,
                          "roofline": {"bound": "mfma", "achieved": round(ach, 1), "peak": 2500.0, "unit": "TFLOP/s",
                                       "frac": round(ach / 2500.0, 4), "traffic": None,
                                       "kernel": "k_linear_quantize_pack"}}))
        return

    if args.fused_matmul:
        (w,) = make_config(args.config)
        # configurations 5 and 3: the linear layer after the activation; configuration 2: the conv
        # activation read as [N*H*W, C] (a pointwise convolution in a channels-last view): a long
        # reduction into a 256 x 256 output
        K = 256 if args.config == 2 else w.x.shape[-1]
        M = w.numel // K
        N = {5: 4096, 3: 3072, 2: 256}.get(args.config, 1024)
        dt = torch.float32 if args.f32 else w.x.dtype
        x = w.x.reshape(-1).to(dev).to(dt)
        bits = int(w.bits[0]) if w.bits.size == 1 else torch.from_numpy(w.bits).to(dev)
        if args.uniform_bits:
            bits = args.uniform_bits
        plan = daf.daf_plan((M, K), w.group_size, bits)
        words = torch.empty(plan.packed_words, dtype=torch.int32, device=dev)
        mn, sc = torch.empty(plan.num_groups, device=dev), torch.empty(plan.num_groups, device=dev)
        daf.daf_quantize_pack(plan, x, w.seed, words, mn, sc)
        gy = (torch.randn(M, N, device=dev) * 0.1).to(dt)
        out = torch.empty(N, K, device=dev)
        ws_bytes = daf.daf_unpack_matmul_workspace_bytes(plan, N, K)
        if ws_bytes < 0:
            print("bench.py: shape not supported by the fused product", file=sys.stderr)
            sys.exit(2)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        xh = torch.empty(M, K, dtype=dt, device=dev)
        out_lib = torch.empty(N, K, dtype=dt, device=dev)

        def timed(fn, reps):
            for _ in range(max(2, args.warmup // 4)):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        def unfused():
            daf.daf_unpack_dequantize(plan, words, mn, sc, xh.view(-1))
            torch.mm(gy.t(), xh, out=out_lib)

        reps = max(3, min(args.steps, 20))
        t_fused = timed(lambda: daf.daf_unpack_matmul_grad_weight(plan, words, mn, sc, gy, out, ws), reps)
        t_unfused = timed(unfused, reps)
        t_mm = timed(lambda: torch.mm(gy.t(), xh, out=out_lib), reps)
        rel = ((out - out_lib.float()).abs().max() / out.abs().max()).item()
        flops = 2.0 * M * N * K
        peak = 157.3 if x.dtype == torch.float32 else 2500.0   # dense MFMA, binary32 / 16-bit formats
        ach = flops / (t_fused * 1e-3) / 1e12
        print(json.dumps({"metric": "weight gradient from the packed activation, TFLOP/s", "value": round(ach, 1),
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": reps, "data": "synthetic", "higher_is_better": True,
                          "dtype": "f32" if args.f32 else {0: "f32", 1: "f16", 2: "bf16"}[w.dtype],
                          "config": {"workload": CONFIG_NAMES[args.config] + f"_grad_weight_N{N}", "M": M, "N": N, "K": K,
                                     "splits_workspace_bytes": ws_bytes},
                          "fused_ms": round(t_fused, 4), "unfused_dequantize_plus_library_mm_ms": round(t_unfused, 4),
                          "library_mm_alone_ms": round(t_mm, 4),
                          "library_mm_TFLOPs": round(flops / (t_mm * 1e-3) / 1e12, 1),
                          "xhat_bytes_never_written": M * K * x.element_size(),
                          "max_rel_diff_vs_library_output": round(rel, 5),
                          "roofline": {"bound": "mfma", "achieved": round(ach, 1), "peak": peak, "unit": "TFLOP/s",
                                       "frac": round(ach / peak, 4), "traffic": None, "kernel": "k_unpack_matmul"}}))
        return

    if args.sweep:
        n = 1 << 27

        def timeit(f, reps=20):
            for _ in range(25):                          # the clocks take tens of milliseconds of load to settle
                f()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                f()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        for dt in (torch.float32, torch.float16, torch.bfloat16):
            xs = [torch.randn(n, device=dev, dtype=torch.float32).to(dt) for _ in range(2)]
            xh = torch.empty_like(xs[0])
            for gs in [int(v) for v in args.sweep_group_sizes.split(",")]:
                G = (n + gs - 1) // gs
                for bits in (1, 2, 4, 8, "mixed"):
                    if bits == "mixed":
                        b = torch.from_numpy(np.random.default_rng(0).choice([1, 2, 4, 8], G).astype(np.uint8)).to(dev)
                        plan = daf.daf_plan((n,), gs, b)
                    else:
                        plan = daf.daf_plan((n,), gs, bits)
                    # packed outputs rotate over more than the memory-side cache holds, so that the
                    # dequantize direction reads them from HBM as a backward pass does
                    packed = plan.packed_words * 4 + 8 * G
                    n_out = max(2, min(40, -(-ROTATE_PACKED_BYTES // packed)))
                    outs = [(torch.empty(plan.packed_words, dtype=torch.int32, device=dev), torch.empty(G, device=dev),
                             torch.empty(G, device=dev)) for _ in range(n_out)]
                    it = [0]

                    def q():
                        daf.daf_quantize_pack(plan, xs[it[0] & 1], 3, *outs[it[0] % n_out])
                        it[0] += 1
                    for _ in range(n_out):
                        q()

                    def d():
                        daf.daf_unpack_dequantize(plan, *outs[it[0] % n_out], xh)
                        it[0] += 1
                    tq = timeit(q)
                    td = timeit(d)
                    alg = n * xs[0].element_size() + plan.packed_words * 4 + G * 8 + (G * 5 if bits == "mixed" else 0)
                    print(json.dumps({"dtype": str(dt)[6:], "group_size": gs, "bits": bits,
                                      "quantize_us": round(tq * 1e3, 1), "quantize_frac": round(alg / (tq * 1e-3) / 8e12, 3),
                                      "dequantize_us": round(td * 1e3, 1),
                                      "dequantize_frac": round(alg / (td * 1e-3) / 8e12, 3)}), flush=True)
                    plan.destroy()
        return

    if args.list_rows:
        res = []
        for shape, gs in (((32, 1024, 768), 768), ((8, 197, 3072), 3072), ((8, 197, 768), 768)):
            n, T = int(np.prod(shape)), 16
            items, keep = [], []
            for i in range(T):
                x = torch.randn(n, device=dev).to(torch.float16)
                G = n // gs
                b = torch.from_numpy(np.random.default_rng(i).choice([1, 2, 4, 8], G).astype(np.uint8)).to(dev)
                p = daf.daf_plan((n,), gs, b)
                items.append((p, x, i, torch.empty(p.packed_words, dtype=torch.int32, device=dev),
                              torch.empty(G, device=dev), torch.empty(G, device=dev)))
                keep.append(b)
            marshalled = daf.quantize_items(items)

            def one_by_one():
                for it in items:
                    daf.daf_quantize_pack(*it)

            def as_list():
                daf.daf_quantize_pack_batch(marshalled)
            row = {"shape": list(shape), "group_size": gs, "tensors": T}
            for name, f in (("one_call_per_tensor_us", one_by_one), ("list_call_us", as_list)):
                for _ in range(10):
                    f()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(30):
                    f()
                e1.record()
                torch.cuda.synchronize()
                row[name] = round(e0.elapsed_time(e1) / 30 * 1e3, 1)
            res.append(row)
            for it in items:
                it[0].destroy()
        print(json.dumps({"metric": "quantize+pack of 16 tensors with one group per row", "unit": "us", "n_gpus": 1,
                          "data": "synthetic", "dtype": "f16", "results": res}))
        return

    if args.output_policy:
        workloads = make_config(args.config)
        in_bytes = sum(w.numel * w.x.element_size() for w in workloads)
        n_sets = 1 if in_bytes >= ROTATE_BYTES else -(-ROTATE_BYTES // in_bytes)
        plans, sets = [], []
        for w in workloads:
            plans.append(daf.daf_plan(tuple(w.x.shape), w.group_size,
                                      int(w.bits[0]) if w.bits.size == 1 else torch.from_numpy(w.bits).to(dev)))
        n_sets = max(n_sets, -(-ROTATE_PACKED_BYTES // sum(4 * p.packed_words + 8 * p.num_groups for p in plans)))
        for _ in range(n_sets):
            bufs = []
            for w, p in zip(workloads, plans):
                b = dict(x=w.x.reshape(-1).to(dev), words=torch.empty(p.packed_words, dtype=torch.int32, device=dev),
                         mn=torch.empty(p.num_groups, device=dev), sc=torch.empty(p.num_groups, device=dev),
                         lo=torch.empty(p.num_groups, device=dev), hi=torch.empty(p.num_groups, device=dev))
                daf.daf_quantize_pack(p, b["x"], w.seed, b["words"], b["mn"], b["sc"])
                bufs.append(b)
            sets.append(bufs)

        def unpack(k):
            for (p, b) in zip(plans, sets[k]):
                daf.daf_unpack_dequantize(p, b["words"], b["mn"], b["sc"], b["x"])

        def reader(k):
            for (p, b) in zip(plans, sets[k]):
                daf.daf_group_minmax(p, b["x"], b["lo"], b["hi"])

        def pair(k):
            for (p, b) in zip(plans, sets[k]):
                daf.daf_unpack_dequantize(p, b["words"], b["mn"], b["sc"], b["x"])
                daf.daf_group_minmax(p, b["x"], b["lo"], b["hi"])

        def timed(fn):
            for i in range(args.warmup):
                fn(i % n_sets)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(args.steps):
                fn(i % n_sets)
            e1.record()
            torch.cuda.synchronize()
            return round(e0.elapsed_time(e1) / args.steps, 4)

        res = {"reader_alone_ms": timed(reader)}
        for cached in (False, True):
            for p in plans:
                p.set_output_cached(cached)
            key = "cached" if cached else "streaming"
            res[key] = {"unpack_alone_ms": timed(unpack), "unpack_then_reader_ms": timed(pair)}
        print(json.dumps({"metric": "unpack+dequantize output store policy", "unit": "ms", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                          "config": {"workload": CONFIG_NAMES[args.config], "tensors": len(workloads),
                                     "buffer_sets": n_sets, "activation_bytes": in_bytes}, **res}))
        return

    if args.fused_relu:
        # pre-activations z = the workload's values with random signs; buffers rotate over > 768 MB
        workloads = make_config(args.config)
        in_bytes = sum(w.numel * w.x.element_size() for w in workloads)
        n_sets = 1 if in_bytes >= ROTATE_BYTES else -(-ROTATE_BYTES // in_bytes)
        gen = torch.Generator().manual_seed(17)
        plans, sets = [], []
        for w in workloads:
            plans.append(daf.daf_plan(tuple(w.x.shape), w.group_size,
                                      int(w.bits[0]) if w.bits.size == 1 else torch.from_numpy(w.bits).to(dev)))
        # (the packed outputs rotate through more than the memory-side cache holds as well, so that
        # the backward kernels read them from HBM)
        n_sets = max(n_sets, -(-ROTATE_PACKED_BYTES // sum(4 * p.packed_words + 8 * p.num_groups for p in plans)))
        for _ in range(n_sets):
            bufs = []
            for w, p in zip(workloads, plans):
                sign = torch.randint(0, 2, (w.numel,), generator=gen, dtype=torch.int8).to(w.x.dtype).mul_(2).sub_(1)
                z = (w.x.reshape(-1) * sign).to(dev)
                bufs.append(dict(z=z, y=torch.empty_like(z),
                                 words=torch.empty(p.packed_words, dtype=torch.int32, device=dev),
                                 mn=torch.empty(p.num_groups, device=dev), sc=torch.empty(p.num_groups, device=dev)))
            sets.append(bufs)

        def fused(k):
            for (w, p, b) in zip(workloads, plans, sets[k]):
                daf.daf_relu_quantize_pack(p, b["z"], w.seed, b["y"], b["words"], b["mn"], b["sc"])

        def separate(k):
            for (w, p, b) in zip(workloads, plans, sets[k]):
                torch.clamp_min(b["z"], 0, out=b["y"])
                daf.daf_quantize_pack(p, b["y"], w.seed, b["words"], b["mn"], b["sc"])

        def timed(fn):
            for i in range(args.warmup):
                fn(i % n_sets)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for i in range(args.steps):
                fn(i % n_sets)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps

        def fused_bwd(k):
            for (w, p, b) in zip(workloads, plans, sets[k]):
                daf.daf_unpack_relu_backward(p, b["words"], b["mn"], b["sc"], b["z"], b["y"])   # z plays grad_y

        def separate_bwd(k):
            for (w, p, b) in zip(workloads, plans, sets[k]):
                daf.daf_unpack_dequantize(p, b["words"], b["mn"], b["sc"], b["y"])
                torch.ops.aten.threshold_backward.grad_input(b["z"], b["y"], 0, grad_input=b["y"])

        t_sep, t_fused = timed(separate), timed(fused)
        t_bsep, t_bfused = timed(separate_bwd), timed(fused_bwd)
        alg = sum(algorithmic_bytes(w, p.packed_words) + w.numel * w.x.element_size()
                  for w, p in zip(workloads, plans))            # z read, y written, words, min, scale
        ach = alg / (t_fused * 1e-3) / 1e9
        ach_b = alg / (t_bfused * 1e-3) / 1e9
        print(json.dumps({"metric": "relu + quantize+pack GB/s of activations", "value": round(in_bytes / t_fused / 1e6, 1),
                          "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                          "higher_is_better": True, "dtype": {0: "f32", 1: "f16", 2: "bf16"}[workloads[0].dtype],
                          "config": {"workload": CONFIG_NAMES[args.config] + "_fused_relu", "tensors": len(workloads),
                                     "buffer_sets": n_sets},
                          "fused_ms": round(t_fused, 4), "separate_relu_then_quantize_ms": round(t_sep, 4),
                          "speedup": round(t_sep / t_fused, 3),
                          "backward_fused_ms": round(t_bfused, 4),
                          "backward_separate_dequantize_then_threshold_ms": round(t_bsep, 4),
                          "backward_speedup": round(t_bsep / t_bfused, 3),
                          "roofline_backward": {"bound": "hbm", "achieved": round(ach_b, 1), "peak": HBM_PEAK_GBPS,
                                                "unit": "GB/s", "frac": round(ach_b / HBM_PEAK_GBPS, 4),
                                                "kernel": "k_unpack_dequantize_tile<..., RELU_BWD>",
                                                "algorithmic_bytes": alg},
                          "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                       "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None,
                                       "kernel": "k_quantize_pack_tile<..., RELU>", "algorithmic_bytes": alg}}))
        return

    if args.config is None and args.group_size is None:
        # The default run: the headline is the largest configuration (the 17-tensor ResNet-18
        # step, 590.9 M elements); the other configurations the 70 % target is stated on ride
        # along as `per_config`, each with both directions' kernel time and roofline fraction.
        out = measure(4, args, daf, torch, np, dev, headline=True)
        out["per_config"] = {}
        for cfg in (2, 3, 5):
            r = measure(cfg, args, daf, torch, np, dev, headline=False)
            out["per_config"][str(cfg)] = r
        print(json.dumps(out))
        return
    print(json.dumps(measure(args.config or 2, args, daf, torch, np, dev, headline=True)))


def measure(cfg, args, daf, torch, np, dev, headline):
    """One configuration: buffers resident in HBM, the timed steps (quantize+pack of the batch,
    then unpack+dequantize), and the kernel time of each direction on one stream for the
    roofline.  headline=False: kernel times and roofline only (a `per_config` record)."""
    from daf_inputs import CONFIG_NAMES, make_config, to_numpy_bits
    workloads = make_config(cfg)
    if args.group_size is not None:
        for w in workloads:
            if w.bits.size != 1:
                print("bench.py: --group-size needs a uniform-width configuration", file=sys.stderr)
                sys.exit(2)
            w.group_size = args.group_size if args.group_size > 0 else ((w.numel + 31) // 32) * 32
    in_bytes = sum(w.numel * w.x.element_size() for w in workloads)
    n_sets = 1 if in_bytes >= ROTATE_BYTES else -(-ROTATE_BYTES // in_bytes)

    # groups longer than 65536 elements (or fewer than 256 groups of a whole number of 4096-element
    # tiles) need their statistics before any element can be quantized: the quantize direction
    # then reads the activation twice (and keeps per-tile statistics in scratch memory owned by
    # the plan, so such a plan serves one call at a time: one plan per buffer set)
    def two_reads(w):
        gs = w.group_size
        return gs > 65536 or (gs > 4096 and gs % 4096 == 0 and w.numel // gs < 256)
    plan_sets = n_sets if any(two_reads(w) for w in workloads) else 1

    # device state: per tensor a plan, and per (set, tensor) its buffers
    plans_by_set, dbits = [], []
    for w in workloads:
        dbits.append(None if w.bits.size == 1 else torch.from_numpy(w.bits).to(dev))
    for _ in range(plan_sets):
        plans_by_set.append([daf.daf_plan(tuple(w.x.shape), w.group_size, int(w.bits[0]) if b is None else b)
                             for w, b in zip(workloads, dbits)])
    plans = plans_by_set[0]
    # The backward pass reads packed words, min and scale that the forward pass wrote long before:
    # they must come from HBM in the timed launches too, so the buffer sets also rotate over more
    # packed bytes than the 256 MB memory-side cache holds (a 14 MB packed tensor would
    # otherwise be served from it and unpack+dequantize would read a quarter faster).
    packed_bytes = sum(4 * p.packed_words + 8 * p.num_groups for p in plans)
    n_sets = max(n_sets, -(-ROTATE_PACKED_BYTES // packed_bytes))
    if plan_sets > 1:
        for _ in range(n_sets - plan_sets):
            plans_by_set.append([daf.daf_plan(tuple(w.x.shape), w.group_size, int(w.bits[0]) if b is None else b)
                                 for w, b in zip(workloads, dbits)])
        plan_sets = n_sets

    def plan_of(k, t):
        return plans_by_set[k % plan_sets][t]
    sets = []
    for s in range(n_sets):
        bufs = []
        for t, (w, p) in enumerate(zip(workloads, plans)):
            x = w.x.reshape(-1).to(dev) if s == 0 else sets[0][t]["x"].clone()
            bufs.append(dict(x=x, words=torch.empty(p.packed_words, dtype=torch.int32, device=dev),
                             mn=torch.empty(p.num_groups, dtype=torch.float32, device=dev),
                             sc=torch.empty(p.num_groups, dtype=torch.float32, device=dev),
                             xh=torch.empty_like(x)))
        sets.append(bufs)
    torch.cuda.synchronize()

    # Tensor t of buffer set k always uses stream (k + t) % n_streams, in both directions and in
    # every step, so its dequantize is ordered after its quantize, and each reuse of a buffer
    # after the previous one, without any cross-stream event.  With more than one stream,
    # independent tensors and independent batches may overlap (the tail of one kernel with the
    # start of the next); the default is one stream, so that a kernel trace of this program
    # shows every kernel alone on the device.
    main = torch.cuda.current_stream()
    streams = [main] + [torch.cuda.Stream() for _ in range(max(0, args.streams - 1))]
    order = list(enumerate(workloads))

    def fork():
        if len(streams) > 1:
            ev = torch.cuda.Event()
            ev.record(main)
            for s in streams[1:]:
                s.wait_event(ev)

    def join():
        for s in streams[1:]:
            ev = torch.cuda.Event()
            ev.record(s)
            main.wait_event(ev)

    # Several tensors per step (the ResNet-18 configuration): the list entry points, one call
    # per direction; the lists are marshalled once.
    batched = len(workloads) > 1
    q_lists = [daf.quantize_items([(plan_of(k, t), sets[k][t]["x"], w.seed, sets[k][t]["words"], sets[k][t]["mn"],
                                    sets[k][t]["sc"]) for t, w in order]) for k in range(n_sets)] if batched else None
    d_lists = [daf.dequantize_items([(plan_of(k, t), sets[k][t]["words"], sets[k][t]["mn"], sets[k][t]["sc"],
                                      sets[k][t]["xh"], None) for t, w in reversed(order)])
               for k in range(n_sets)] if batched else None

    def quantize_all(k, single=False):
        if batched:
            daf.daf_quantize_pack_batch(q_lists[k], stream=main if single else streams[k % len(streams)])
            return
        for t, w in order:
            b = sets[k][t]
            daf.daf_quantize_pack(plan_of(k, t), b["x"], w.seed, b["words"], b["mn"], b["sc"],
                                  stream=main if single else streams[(k + t) % len(streams)])

    def dequantize_all(k, single=False):
        if batched:
            daf.daf_unpack_dequantize_batch(d_lists[k], stream=main if single else streams[k % len(streams)])
            return
        for t, w in reversed(order):
            b = sets[k][t]
            daf.daf_unpack_dequantize(plan_of(k, t), b["words"], b["mn"], b["sc"], b["xh"],
                                      stream=main if single else streams[(k + t) % len(streams)])

    def step(i):
        # forward order, then reverse order (a training step saves, then restores backwards)
        quantize_all(i % n_sets)
        dequantize_all(i % n_sets)

    fork()
    for i in range(args.warmup):
        step(i)
    join()
    torch.cuda.synchronize()
    ms_per_step = None
    if headline:
        t0 = time.perf_counter()
        fork()
        for i in range(args.steps):
            step(args.warmup + i)
        join()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps

    # Kernel time per direction, for the roofline: the launches of one direction back to back on
    # ONE stream (rotating over the buffer sets, no overlap between kernels), bracketed by HIP
    # events on that stream, one pair per batch of launches, so that the few microseconds an
    # event pair costs are not charged to every launch.
    def kernel_pass(direction, batch, n_batches):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_batches + 1)]
        evs[0].record()
        r = 0
        for b in range(n_batches):
            for _ in range(batch):
                if direction == "q":
                    quantize_all(r % n_sets, single=True)
                else:
                    dequantize_all(r % n_sets, single=True)
                r += 1
            evs[b + 1].record()
        torch.cuda.synchronize()
        per = sorted(evs[b].elapsed_time(evs[b + 1]) / batch for b in range(n_batches))
        return {"median": per[len(per) // 2], "min": per[0], "mean": sum(per) / len(per)}

    batch = max(10, n_sets) if len(workloads) == 1 else 1
    n_batches = max(5, -(-args.steps // batch))
    kernel_pass("q", n_sets, 1)
    qk = kernel_pass("q", batch, n_batches)
    kernel_pass("d", n_sets, 1)
    dk = kernel_pass("d", batch, n_batches)
    qk_ms, dk_ms = qk["median"], dk["median"]
    alg = sum(algorithmic_bytes(w, p.packed_words) for w, p in zip(workloads, plans))
    alg_q = alg + sum(w.numel * w.x.element_size() for w in workloads if two_reads(w))
    gs0 = workloads[0].group_size
    q_kernel_name = ("k_quantize_pack_tile" if gs0 & (gs0 - 1) == 0 and gs0 <= 4096 or two_reads(workloads[0])
                     else "k_quantize_pack_units" if gs0 <= 4096 else "k_quantize_pack_long")
    if batched:
        q_kernel_name += "_batch"
    pow2 = gs0 > 0 and gs0 & (gs0 - 1) == 0
    fp32_8bit = workloads[0].x.dtype == torch.float32 and workloads[0].bits.size == 1 and int(workloads[0].bits[0]) == 8
    if pow2 and gs0 <= 4096:
        d_kernel_name = "k_unpack_dequantize_tile" + ("_batch" if batched else "")
    elif not pow2 and 64 <= gs0 <= 32768 and not batched and not fp32_8bit:
        d_kernel_name = "k_unpack_dequantize_tile_any"
    else:
        d_kernel_name = "k_unpack_dequantize_chunk" + ("_batch" if batched else "")

    traffic = QUOTED_TRAFFIC.get(cfg) if args.group_size is None else None

    def roof(ms, which, nbytes):
        ach = nbytes / (ms * 1e-3) / 1e9
        r = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
             "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": traffic[which] if traffic else None}
        if traffic:
            r["traffic_source"] = "quoted, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in " + traffic[2]
        return r

    dt_name = {0: "f32", 1: "f16", 2: "bf16"}[workloads[0].dtype]
    rec = {
        "workload": CONFIG_NAMES[cfg], "dtype": dt_name, "tensors": len(workloads),
        "elements": sum(w.numel for w in workloads), "group_size": workloads[0].group_size, "buffer_sets": n_sets,
        "quantize_pack": {"kernel_ms": round(qk_ms, 4), "kernel_ms_min": round(qk["min"], 4),
                          "kernel_ms_mean": round(qk["mean"], 4),
                          "input_GBps": round(in_bytes / qk_ms / 1e6, 1), "algorithmic_bytes": alg_q,
                          "launches": 1 if batched else len(workloads)},
        "unpack_dequantize": {"kernel_ms": round(dk_ms, 4), "kernel_ms_min": round(dk["min"], 4),
                              "kernel_ms_mean": round(dk["mean"], 4),
                              "output_GBps": round(in_bytes / dk_ms / 1e6, 1), "algorithmic_bytes": alg,
                              "launches": 1 if batched else len(workloads)},
        "roofline": dict(roof(qk_ms, 0, alg_q), kernel=q_kernel_name),
        "roofline_unpack_dequantize": dict(roof(dk_ms, 1, alg), kernel=d_kernel_name),
    }
    if not headline:
        for ps in plans_by_set:
            for p in ps:
                p.destroy()
        return rec

    value = 2 * in_bytes / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "quantize+pack and unpack+dequantize GB/s of activations",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dt_name,
        "data": "synthetic", "config": {"workload": CONFIG_NAMES[cfg], "tensors": len(workloads),
                                        "elements": rec["elements"], "group_size": rec["group_size"],
                                        "buffer_sets": n_sets, "streams": len(streams)},
        "quantize_pack": rec["quantize_pack"], "unpack_dequantize": rec["unpack_dequantize"],
        "roofline": rec["roofline"], "roofline_unpack_dequantize": rec["roofline_unpack_dequantize"],
    }
    del sets, q_lists, d_lists
    torch.cuda.empty_cache()

    if not args.no_cpu_baseline:
        from oracle import daf_oracle as orc
        # The oracle as it stands, one thread, quantize+pack then unpack+dequantize, on the first
        # tensors of the same workload up to ~1.2 GB of input (~10-20 s of CPU work), one pass.
        budget, sample, done = 1200 << 20, [], 0
        for w in workloads:
            if sample and done + w.numel * w.x.element_size() > budget:
                break
            sample.append(w)
            done += w.numel * w.x.element_size()
        t = time.perf_counter()
        for w in sample:
            xb = to_numpy_bits(w.x)
            ow, omn, osc, _ = orc.quantize_pack(xb, w.dtype, w.group_size, w.bits, w.seed)
            orc.unpack_dequantize(ow, omn, osc, w.bits, w.numel, w.group_size, w.dtype)
            del ow, omn, osc
        best = time.perf_counter() - t
        out["cpu_baseline"] = {"value": round(2 * done / best / 1e9, 4), "unit": "GB/s", "cores": 1,
                               "kind": "oracle", "seconds": round(best, 2),
                               "sample": f"the first {len(sample)} of {len(workloads)} tensors, {done} input bytes, "
                                         "quantize+pack then unpack+dequantize, one pass"}
        # the same oracle functions over disjoint group ranges (groups are independent once
        # the offsets are known), one range per host thread: a second reported baseline
        import concurrent.futures as cf
        n_thr = max(1, min(len(os.sched_getaffinity(0)), 16))
        prepared = []
        for w in sample:
            xb = to_numpy_bits(w.x).reshape(-1)
            off, total = orc.plan(w.numel, w.group_size, w.bits)
            G = orc.num_groups(w.numel, w.group_size)
            prepared.append((w, xb, off, G, np.empty(total, np.uint32), np.empty(G, np.float32),
                             np.empty(G, np.float32), np.empty(w.numel, xb.dtype)))

        def one_range(args_):
            (w, xb, off, G, ow, omn, osc, oxh), g0, g1 = args_
            orc.quantize_pack_range(xb, w.dtype, w.group_size, w.bits, off, w.seed, g0, g1, ow, omn, osc)
            orc.unpack_dequantize_range(ow, omn, osc, w.bits, off, w.numel, w.group_size, g0, g1, oxh, w.dtype)

        jobs = []
        for p_ in prepared:
            G = p_[3]
            cuts = [G * i // n_thr for i in range(n_thr + 1)]
            jobs += [(p_, cuts[i], cuts[i + 1]) for i in range(n_thr) if cuts[i + 1] > cuts[i]]
        best_mt = float("inf")
        with cf.ThreadPoolExecutor(max_workers=n_thr) as ex:
            for _ in range(2):
                t = time.perf_counter()
                list(ex.map(one_range, jobs))
                best_mt = min(best_mt, time.perf_counter() - t)
        out["cpu_baseline_all_cores"] = {"value": round(2 * done / best_mt / 1e9, 4), "unit": "GB/s",
                                         "cores": n_thr, "kind": "oracle", "seconds": round(best_mt, 2),
                                         "sample": "same sample, groups split into one range per thread, best of 2"}
    for ps in plans_by_set:
        for p in ps:
            p.destroy()
    return out


if __name__ == "__main__":
    main()
