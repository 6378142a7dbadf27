"""Benchmark of the LBP-WHT linear-layer backward (gx + gW) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--rank R] [--order l1|linf]

A step is one whole pass of the hot path through the C ABI: projection of gy and x, the two
low-rank products and the reverse projection of gx (Algorithm 1), on synthetic ViT-shaped inputs
that are already resident in HBM.  The default workload is the ViT-B MLP fc1 backward (N=64,
16x16 tokens, 768->3072, patch 8, r=8 low-pass bases, bf16 tensors with fp32 accumulation).
Consecutive steps rotate over several distinct sets of buffers so that the working set exceeds the
256 MB last-level cache (cache-cold timing); --warm-cache reuses one set.

Prints ONE JSON line.  `value` is the Table-1 FLOPs of LBP-WHT (projection + low-rank products +
reverse projection, per patch, summed over the batch) per second.  The line also carries:
  full_bp_ms / speedup_vs_full_bp   the same-style exact backward (Eq. 2) from this library,
  library_gemm_full_bp_ms           the two products through torch.matmul (the vendor GEMM library)
                                    as a second opinion on the comparison point,
  best_of_both_full_bp_ms           the strongest exact backward on hand: each product from whichever of
                                    this library and the vendor's is faster (each timed alone),
  library_gemm_lowrank_products_ms  the two low-rank products through torch.matmul, to set beside
                                    stages.products_us,
  preprojected_x_ms_per_step        lbp_wht_backward_preprojected: x^ kept from the forward pass,
  stages                            each part of a call timed by itself, back to back (projection; the two
                                    products as the call launches them; each product launched alone),
  roofline                          the kernel that takes the larger share of a step: the two products
                                    (one grouped launch at the default workload; `kernel` says what the
                                    planner launches at this rank; bf16 MFMA: algorithmic FLOPs / average
                                    duration) or the projection of gy and x (HBM: algorithmic bytes /
                                    average duration); roofline_second is the other one; `traffic` is
                                    filled in only where profiles/ holds counters for this workload and rank,
  warm_cache_ms_per_step            the same step on one buffer set over and over (cache-warm), labelled,
  cpu_baseline                      the CPU oracle timed on this machine's host cores (all threads; beside it one
                                    thread, and the oracle's exact backward).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def lbp_flops(wl, r):
    """Table 1 per patch (L = patch^2 tokens), summed over the patches of the batch."""
    L = wl.patch * wl.patch
    per_patch = (wl.Cin + wl.Cout) * L * r + 4 * wl.Cin * wl.Cout * r + wl.Cin * L * r
    return float(per_patch) * wl.patches + 4.0 * wl.Cin * wl.Cout * wl.N * wl.extra      # tokens outside the grid: Eq. 2


def full_bp_flops(wl):
    return 4.0 * wl.Cin * wl.Cout * wl.tokens


def read_traffic(name, r, order):
    """HBM bytes per launch of a kernel from the committed rocprofv3 counter summary (profiles/<name>),
    or None when there is none for this workload, rank and basis order."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    matches = False
    for line in open(path):
        if line.startswith("measured_at"):
            matches = line.split()[1:] == [f"rank={r}", f"order={order}"]
        if line.startswith("traffic_bytes_per_launch"):
            return float(line.split()[1]) if matches else None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg2_vitb_fc1")
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--order", default="l1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-library-gemm", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay timing")
    ap.add_argument("--warm-cache", action="store_true", help="reuse one buffer set (cache-warm timing)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    import torch

    from paper_2309_15275_amd import binding, workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    wl = workloads.WORKLOADS[args.workload]
    r = args.rank or wl.ranks[0]
    idx = binding.select_bases(wl.patch, r, args.order)
    esz = 4 if wl.dtype == "f32" else 2

    # token-sequence workloads ([N, extra + H*W, C], a class token in front of the grid) go through
    # the *_tokens entry points; the exact backward sees the same tokens as one long row of a grid
    seq = wl.extra > 0
    T = wl.H * wl.W + wl.extra
    host = workloads.make_token_inputs(wl, wl.extra) if seq else workloads.make_inputs(wl)

    def dev(a):
        if wl.dtype == "f32":
            return torch.from_numpy(a).cuda()
        return torch.from_numpy(workloads.bf16_bits(a).reshape(a.shape).view(np.int16)).cuda().view(torch.bfloat16)

    base = {k: dev(v) for k, v in host.items()}
    set_bytes = sum(t.numel() * t.element_size() for t in base.values()) + base["x"].numel() * esz \
        + base["w"].numel() * 4
    n_sets = 1 if args.warm_cache else max(2, int(np.ceil(600e6 / set_bytes)))
    sets = []
    for i in range(n_sets):
        s = {k: (v if i == 0 else v.clone()) for k, v in base.items()}
        s["gx"] = torch.empty_like(s["x"])
        s["gW"] = torch.empty(s["w"].shape, dtype=torch.float32, device="cuda")
        sets.append(s)

    grid = (wl.H, wl.W)

    def as_grid(t):      # [N, T, C] -> [N, 1, T, C] for the entry points that take grids
        return t.view(wl.N, 1, T, t.shape[-1]) if seq else t

    def lbp_step(i):
        s = sets[i % n_sets]
        if seq:
            binding.lbp_wht_backward_tokens(s["x"], s["gy"], s["w"], grid, wl.patch, idx, gx=s["gx"], gW=s["gW"])
        else:
            binding.lbp_wht_backward(s["x"], s["gy"], s["w"], wl.patch, idx, gx=s["gx"], gW=s["gW"])

    def full_step(i):
        s = sets[i % n_sets]
        binding.full_bp_backward(as_grid(s["x"]), as_grid(s["gy"]), s["w"], gx=as_grid(s["gx"]), gW=s["gW"])

    def lib_step(i):
        s = sets[i % n_sets]
        G = s["gy"].view(-1, wl.Cout)
        torch.matmul(G, s["w"], out=s["gx"].view(-1, wl.Cin))
        torch.matmul(G.t(), s["x"].view(-1, wl.Cin))      # allocates its result: the library's habit, not timed apart

    def timed(fn, steps, warmup):
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            fn(warmup + i)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return e0.elapsed_time(e1) / steps, wall_ms / steps

    if seq:      # no two-tensor entry point for sequences: one projection call per tensor
        proj_bufs = [(binding.wht_project_tokens(s["x"], grid, wl.patch, idx),
                      binding.wht_project_tokens(s["gy"], grid, wl.patch, idx)) for s in sets]
    else:
        proj_bufs = [binding.wht_project_pair(s["x"], s["gy"], wl.patch, idx) for s in sets]

    def proj_step(i):
        s, (xr, gyr) = sets[i % n_sets], proj_bufs[i % n_sets]
        if seq:
            binding.wht_project_tokens(s["x"], grid, wl.patch, idx, out=xr)
            binding.wht_project_tokens(s["gy"], grid, wl.patch, idx, out=gyr)
        else:
            binding.wht_project_pair(s["x"], s["gy"], wl.patch, idx, x_r=xr, gy_r=gyr)

    def pre_step(i):
        s, (xr, _) = sets[i % n_sets], proj_bufs[i % n_sets]
        if seq:
            binding.lbp_wht_backward_tokens_preprojected(xr, s["gy"], s["w"], grid, wl.patch, idx, gx=s["gx"], gW=s["gW"])
        else:
            binding.lbp_wht_backward_preprojected(xr, s["gy"], s["w"], wl.patch, idx, gx=s["gx"], gW=s["gW"])

    def prod_step(i):      # the products alone, from projected tensors (grid workloads)
        s, (xr, gyr) = sets[i % n_sets], proj_bufs[i % n_sets]
        binding.lbp_wht_products(xr, gyr, s["w"], (wl.N, wl.H, wl.W), wl.patch, idx, gx=s["gx"], gW=s["gW"])

    ms_lbp, wall_lbp = timed(lbp_step, args.steps, args.warmup)
    # the cache-warm number beside it, labelled: one buffer set over and over
    ms_warm = None if args.warm_cache else timed(lambda i: lbp_step(0), max(20, args.steps // 2), max(5, args.warmup // 2))[0]
    # the same steps recorded once into a HIP graph (one step per buffer set) and replayed: what a
    # training loop that captures its backward pass sees; launch gaps between the kernels shrink
    ms_graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(n_sets):
                lbp_step(i)
        reps = max(1, args.steps // n_sets)
        ms_graph, _ = timed(lambda i: graph.replay(), reps, max(1, args.warmup // n_sets))
        ms_graph /= n_sets
    # the variant that keeps x^ from the forward pass (never reads x)
    ms_pre, _ = timed(pre_step, args.steps, args.warmup)
    # the dominant kernel by itself, back to back on the launch stream (same rotation of buffers)
    ms_proj, _ = timed(proj_step, args.steps, args.warmup)
    ms_prod = None if seq else timed(prod_step, args.steps, args.warmup)[0]
    ms_full, _ = timed(full_step, max(10, args.steps // 4), max(3, args.warmup // 4))
    ms_lib = ms_lib_lowrank = ms_best_full = None
    if not args.no_library_gemm:
        ms_lib, _ = timed(lib_step, max(10, args.steps // 4), max(3, args.warmup // 4))
        # the strongest exact backward on hand: each of its two products from whichever of this
        # library and the vendor's is faster, each timed alone
        n_q, w_q = max(10, args.steps // 4), max(3, args.warmup // 4)

        def own_gx(i):
            s = sets[i % n_sets]
            binding.full_bp_backward(as_grid(s["x"]), as_grid(s["gy"]), s["w"], gx=as_grid(s["gx"]), want_gw=False)

        def own_gw(i):
            s = sets[i % n_sets]
            binding.full_bp_backward(as_grid(s["x"]), as_grid(s["gy"]), s["w"], gW=s["gW"], want_gx=False)

        def lib_gx(i):
            s = sets[i % n_sets]
            torch.matmul(s["gy"].view(-1, wl.Cout), s["w"], out=s["gx"].view(-1, wl.Cin))

        def lib_gw(i):
            s = sets[i % n_sets]
            torch.matmul(s["gy"].view(-1, wl.Cout).t(), s["x"].view(-1, wl.Cin))

        full_parts = {"own_gx_ms": timed(own_gx, n_q, w_q)[0], "own_gw_ms": timed(own_gw, n_q, w_q)[0],
                      "library_gx_ms": timed(lib_gx, n_q, w_q)[0], "library_gw_ms": timed(lib_gw, n_q, w_q)[0]}
        ms_best_full = min(full_parts["own_gx_ms"], full_parts["library_gx_ms"]) + \
            min(full_parts["own_gw_ms"], full_parts["library_gw_ms"])
        if not seq:
            # the two LOW-RANK products through the vendor GEMM library, from the projected tensors
            # (no reverse projection, no 1/p^2): what a library call costs on shapes this small
            lr_out = [torch.empty((xr.shape[0], wl.Cin), dtype=xr.dtype, device="cuda") for xr, _ in proj_bufs]

            def lib_lowrank_step(i):
                s, (xr, gyr) = sets[i % n_sets], proj_bufs[i % n_sets]
                torch.matmul(gyr, s["w"], out=lr_out[i % n_sets])
                torch.matmul(gyr.t(), xr)

            ms_lib_lowrank, _ = timed(lib_lowrank_step, max(20, args.steps // 2), max(5, args.warmup // 2))

    # where the time of a call goes: each part timed by itself, back to back on the launch stream
    # (the projection loop and the products loop above; here the two products launched alone)
    ms_gw = ms_gx = None
    if not seq:
        def gw_step(i):
            s, (xr, gyr) = sets[i % n_sets], proj_bufs[i % n_sets]
            binding.lbp_wht_products(xr, gyr, s["w"], (wl.N, wl.H, wl.W), wl.patch, idx, gW=s["gW"], want_gx=False)

        def gx_step(i):
            s, (xr, gyr) = sets[i % n_sets], proj_bufs[i % n_sets]
            binding.lbp_wht_products(xr, gyr, s["w"], (wl.N, wl.H, wl.W), wl.patch, idx, gx=s["gx"], want_gw=False)

        ms_gw, _ = timed(gw_step, max(20, args.steps // 2), max(5, args.warmup // 2))
        ms_gx, _ = timed(gx_step, max(20, args.steps // 2), max(5, args.warmup // 2))

    if args.calibration_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()

    flops = lbp_flops(wl, r)
    Mr = wl.patches * r + wl.N * wl.extra
    # dominant kernel: the projection launch.  Algorithmic bytes: read gy and x once, write the r/p^2
    # fraction of each (and the tokens outside the grid as they are).
    proj_bytes = esz * (wl.tokens + Mr) * (wl.Cout + wl.Cin)
    proj_gbs = proj_bytes / (ms_proj * 1e-3) / 1e9
    roof_proj = {"bound": "hbm", "kernel": "projection of gy and x (one launch per tensor, token sequences)" if seq
                 else "projection of gy and x (one launch)",
                "achieved": round(proj_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(proj_gbs / HBM_PEAK_GBS, 4),
                "traffic": read_traffic(f"wht_project_{wl.name}_hbm_traffic.txt", r, args.order),
                "algorithmic_bytes": proj_bytes, "avg_launch_us": round(ms_proj * 1e3, 2)}
    gemm_flops = 2.0 * Mr * wl.Cin * wl.Cout
    # what the planner launches for the products of this call (tiles, one launch or several)
    shape = binding.LbpShape(wl.N, wl.H, wl.W, wl.Cin, wl.Cout, binding.LBP_F32 if wl.dtype == "f32" else binding.LBP_BF16,
                             binding.LBP_F32)
    plan_text = binding.describe_plan(shape, wl.patch, idx, extra=wl.extra)
    plan_products = plan_text.split("products: ", 1)[-1].split("; workspace", 1)[0]
    # the two products (one grouped launch where the planner groups them; with the reverse projection
    # in the epilogue where it can be fused): 2 * M_r * Cin * Cout FLOPs each against the dense bf16
    # (fp32: vector fp32) peak; timed back to back from projected tensors on the launch stream
    roof_prod = None
    if ms_prod is not None:
        peak = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else 157.3
        tf = 2.0 * gemm_flops / (ms_prod * 1e-3) / 1e12
        roof_prod = {"bound": "mfma" if wl.dtype == "bf16" else "alu",
                     "kernel": "the two products of a call, g^y W with the reverse projection of Eq. 7 and g^y^T x^ (" + plan_products + ")",
                     "achieved": round(tf, 1), "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4),
                     "traffic": read_traffic(f"gemm_products_{wl.name}_hbm_traffic.txt", r, args.order),
                     "algorithmic_flops": 2.0 * gemm_flops, "avg_launch_us": round(ms_prod * 1e3, 2)}
        # the other candidate bound: operands read once, outputs written once
        prod_bytes = esz * (Mr * (wl.Cin + wl.Cout) + wl.Cin * wl.Cout + wl.tokens * wl.Cin) + 4 * wl.Cin * wl.Cout
        roof_prod["algorithmic_bytes"] = prod_bytes
        roof_prod["frac_of_hbm_peak"] = round(prod_bytes / (ms_prod * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    # `roofline` is the kernel that takes the larger share of a step, `roofline_second` the other
    if roof_prod is not None and ms_prod > ms_proj:
        roofline, roofline_second = roof_prod, roof_proj
    else:
        roofline, roofline_second = roof_proj, roof_prod
    stages = None if seq else {
        "projection_us": round(ms_proj * 1e3, 2),
        "products_us": round(ms_prod * 1e3, 2),
        "gw_product_alone_us": round(ms_gw * 1e3, 2),
        "gx_product_reverse_projection_alone_us": round(ms_gx * 1e3, 2),
        "gw_product_alone_frac_of_mfma_peak": round(gemm_flops / (ms_gw * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "gx_product_alone_frac_of_mfma_peak": round(gemm_flops / (ms_gx * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
    }

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: as many leading images as keep the oracle's work near 20 GFLOP
        n_s = int(max(1, min(wl.N, round(wl.N * 20e9 / max(flops, 1.0)))))
        sample = {k: (v[:n_s] if k != "w" else v) for k, v in host.items()}
        wl_s = workloads.scaled(wl, N=n_s)
        best = 1e30
        for _ in range(2):
            t0 = time.perf_counter()
            if seq:
                oracle.lbp_wht_backward_tokens(sample["x"], sample["gy"], sample["w"], grid, wl.patch, np.asarray(idx))
            else:
                oracle.lbp_wht_backward_padded(sample["x"], sample["gy"], sample["w"], wl.patch, np.asarray(idx))
            best = min(best, time.perf_counter() - t0)
        threads = oracle.max_threads()
        cpu = {"value": round(lbp_flops(wl_s, r) / best / 1e12, 6), "unit": "TFLOP/s",
               "cores": threads, "kind": "oracle",
               "sample": f"first {n_s} of {wl.N} images of the same workload, best of 2 calls, {best:.2f} s each",
               "ms_per_step_scaled_to_full": round(best * 1e3 * wl.N / n_s, 1)}
        # beside it: the same oracle call on one thread, and the oracle's exact backward (Eq. 2) on
        # all threads, each on a sample bounded to a few seconds, scaled to the full batch
        n_1 = max(1, n_s // 8)
        one = {k: (v[:n_1] if k != "w" else v) for k, v in host.items()}
        oracle.set_threads(1)
        t0 = time.perf_counter()
        if seq:
            oracle.lbp_wht_backward_tokens(one["x"], one["gy"], one["w"], grid, wl.patch, np.asarray(idx))
        else:
            oracle.lbp_wht_backward_padded(one["x"], one["gy"], one["w"], wl.patch, np.asarray(idx))
        t_one = time.perf_counter() - t0
        oracle.set_threads(threads)
        n_f = int(max(1, min(wl.N, round(wl.N * 10e9 / max(full_bp_flops(wl), 1.0)))))
        fb = {k: (v[:n_f].reshape(n_f, 1, -1, v.shape[-1]) if k != "w" else v) for k, v in host.items()}
        t0 = time.perf_counter()
        oracle.full_bp_backward(fb["x"], fb["gy"], fb["w"])
        t_full = time.perf_counter() - t0
        cpu["single_thread_ms_per_step_scaled_to_full"] = round(t_one * 1e3 * wl.N / n_1, 1)
        cpu["full_bp_oracle_ms_per_step_scaled_to_full"] = round(t_full * 1e3 * wl.N / n_f, 1)
        cpu["side_samples"] = f"one thread: first {n_1} images, {t_one:.2f} s; exact backward on {threads} threads: first {n_f} images, {t_full:.2f} s"

    out = {
        "metric": "lbp_wht_linear_backward_tflops",
        "value": round(flops / (ms_lbp * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_lbp, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "grid": [wl.H, wl.W], "extra_tokens": wl.extra, "Cin": wl.Cin,
                   "Cout": wl.Cout,
                   "patch": wl.patch, "r": r, "order": args.order,
                   "cache": "warm" if args.warm_cache else f"cold ({n_sets} rotating buffer sets)"},
        "lbp_flops_per_step": flops,
        "bp_equivalent_tflops": round(full_bp_flops(wl) / (ms_lbp * 1e-3) / 1e12, 3),
        "full_bp_ms": round(ms_full, 5),
        "full_bp_tflops": round(full_bp_flops(wl) / (ms_full * 1e-3) / 1e12, 3),
        "speedup_vs_full_bp": round(ms_full / ms_lbp, 3),
        "library_gemm_full_bp_ms": None if ms_lib is None else round(ms_lib, 5),
        "speedup_vs_library_gemm_full_bp": None if ms_lib is None else round(ms_lib / ms_lbp, 3),
        "best_of_both_full_bp_ms": None if ms_best_full is None else round(ms_best_full, 5),
        "speedup_vs_best_of_both_full_bp": None if ms_best_full is None else round(ms_best_full / ms_lbp, 3),
        "full_bp_products_alone_ms": None if ms_best_full is None else {k: round(v, 5) for k, v in full_parts.items()},
        "library_gemm_lowrank_products_ms": None if ms_lib_lowrank is None else round(ms_lib_lowrank, 5),
        "preprojected_x_ms_per_step": round(ms_pre, 5),
        "preprojected_x_speedup_vs_full_bp": round(ms_full / ms_pre, 3),
        "graph_replay_ms_per_step": None if ms_graph is None else round(ms_graph, 5),
        "host_wall_ms_per_step": round(wall_lbp, 5),
        "warm_cache_ms_per_step": None if ms_warm is None else round(ms_warm, 5),
        "stages": stages,
        "roofline": roofline,
        "roofline_second": roofline_second,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
