"""Benchmark of the LBP-WHT linear-layer backward (gx + gW) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--rank R]

A step is one whole pass of the hot path: projection of gy and x, the two low-rank products and
the reverse projection of gx (Algorithm 1), through the C ABI, on synthetic ViT-shaped inputs
that are already resident in HBM.  The default workload is the ViT-B MLP fc1 backward
(N=64, 16x16 tokens, 768->3072, patch 8, r=8, bf16 with fp32 accumulation).  Consecutive steps
rotate over several distinct sets of buffers so that the working set exceeds the 256 MB
last-level cache (cache-cold timing).

Prints ONE JSON line.  `value` is Table-1 FLOPs of LBP-WHT (projection + low-rank products +
reverse projection) per second of wall time; the line also carries the time of the same-style
full-rank backward (Eq. 2), the speedup over it, the roofline of the dominant kernel (the
projection of gy, HBM-bound) and the CPU oracle timed on the host cores on a bounded sample.
"""
import argparse
import json
import sys
import time

import numpy as np


def lbp_flops(wl, r):
    """Table 1 per patch (L = patch^2 tokens), summed over the patches of the batch."""
    L = wl.patch * wl.patch
    per_patch = (wl.Cin + wl.Cout) * L * r + 4 * wl.Cin * wl.Cout * r + wl.Cin * L * r
    return float(per_patch) * wl.patches


def full_bp_flops(wl):
    return 4.0 * wl.Cin * wl.Cout * wl.tokens


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2_vitb_fc1")
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--order", default="l1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--warm-cache", action="store_true", help="reuse one buffer set (cache-warm timing)")
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
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    esz = 4 if wl.dtype == "f32" else 2

    host = workloads.make_inputs(wl)

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

    def lbp_step(i):
        s = sets[i % n_sets]
        binding.lbp_wht_backward(s["x"], s["gy"], s["w"], wl.patch, idx, gx=s["gx"], gW=s["gW"])

    def full_step(i):
        s = sets[i % n_sets]
        binding.full_bp_backward(s["x"], s["gy"], s["w"], gx=s["gx"], gW=s["gW"])

    proj_out = [binding.wht_project(s["gy"], wl.patch, idx) for s in sets]

    def proj_step(i):
        binding.wht_project(sets[i % n_sets]["gy"], wl.patch, idx, out=proj_out[i % n_sets])

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

    ms_lbp, wall_lbp = timed(lbp_step, args.steps, args.warmup)
    ms_full, _ = timed(full_step, max(5, args.steps // 5), max(2, args.warmup // 5))
    ms_proj, _ = timed(proj_step, args.steps, args.warmup)

    flops = lbp_flops(wl, r)
    # dominant kernel: projection of gy.  Algorithmic bytes: read M*Cout once, write M_r*Cout.
    proj_bytes = esz * (wl.tokens + wl.patches * r) * wl.Cout
    achieved = proj_bytes / (ms_proj * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "wht_project(gy)", "achieved": round(achieved, 1), "peak": 8000.0,
                "unit": "GB/s", "frac": round(achieved / 8000.0, 4), "traffic": None,
                "algorithmic_bytes": proj_bytes, "avg_launch_us": round(ms_proj * 1e3, 2)}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_s = max(1, wl.N // 8)
        sample = {k: (v[:n_s] if k != "w" else v) for k, v in host.items()}
        wl_s = workloads.scaled(wl, N=n_s)
        t0 = time.perf_counter()
        oracle.lbp_wht_backward(sample["x"], sample["gy"], sample["w"], wl.patch, np.asarray(idx))
        dt = time.perf_counter() - t0
        cpu = {"value": round(lbp_flops(wl_s, r) / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.max_threads(),
               "kind": "oracle", "sample": f"first {n_s} of {wl.N} images of the same workload, one call, {dt:.2f} s",
               "ms_per_step_scaled_to_full": round(dt * 1e3 * wl.N / n_s, 1)}

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
        "config": {"workload": wl.name, "N": wl.N, "grid": [wl.H, wl.W], "Cin": wl.Cin, "Cout": wl.Cout,
                   "patch": wl.patch, "r": r, "order": args.order,
                   "cache": "warm" if args.warm_cache else f"cold ({n_sets} rotating buffer sets)"},
        "lbp_flops_per_step": flops,
        "bp_equivalent_tflops": round(full_bp_flops(wl) / (ms_lbp * 1e-3) / 1e12, 3),
        "full_bp_ms": round(ms_full, 5),
        "full_bp_tflops": round(full_bp_flops(wl) / (ms_full * 1e-3) / 1e12, 3),
        "speedup_vs_full_bp": round(ms_full / ms_lbp, 3),
        "host_wall_ms_per_step": round(wall_lbp, 5),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
