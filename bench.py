"""Benchmark of the LBP-WHT linear-layer backward (gx + gW) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--rank R] [--order l1|linf]

A step is one whole pass of the hot path through the C ABI: projection of gy and x, the two
low-rank products and the reverse projection of gx (Algorithm 1), on synthetic ViT-shaped inputs
that are already resident in HBM.  The default workload is the ViT-B MLP fc1 backward (N=64,
16x16 tokens, 768->3072, patch 8, r=8 low-pass bases, bf16 tensors with fp32 accumulation).
Consecutive steps rotate over several distinct sets of buffers so that the working set exceeds the
256 MB last-level cache (cache-cold timing); --warm-cache reuses one set.

Timing protocol.  `ms_per_step` (and `value`) is the contract's loop: W untimed steps, then exactly
K steps between two events, bracketed by device synchronisation.  Every other figure -- the stages,
the roofline kernels, the comparison points, the sweep -- comes from at least 100 launches whatever
K is, timed in batches of 10 back-to-back launches, every batch between its own pair of events on
the launch stream, and is the MEDIAN over the batches of the time per launch.  (An event between
two launches costs about 2 us here: beside the roofline kernels `single_launch_us` gives the median
with every launch between its own events, for comparison.)  All calls go to the library
through argument lists built once per buffer set, so the host side of a launch is a few
microseconds and the loops are bound by the GPU.

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
  stages                            each part of a call timed by itself (projection; the two products as the
                                    call launches them; each product launched alone),
  roofline                          the kernel that takes the larger share of a step: the two products
                                    (one grouped launch at the default workload; `kernel` says what the
                                    planner launches at this rank; bf16 MFMA: algorithmic FLOPs / median
                                    launch duration) or the projection of gy and x (HBM: algorithmic bytes /
                                    median launch duration); roofline_second is the other one; `traffic` is
                                    the stored rocprofv3 counter reading under profiles/ for this workload and
                                    rank (`traffic_source` names the file), null where there is none,
  warm_cache_ms_per_step            the same step on one buffer set over and over (cache-warm), labelled,
  sweep                             one row per benchmark configuration, rank and basis order: time of the
                                    low-rank backward, of the exact backward, their ratio, and the roofline
                                    fractions of the projection (of the 8 TB/s HBM peak) and of the products (of
                                    the dense bf16 matrix-core peak; fp32 rows: of the 157.3 TFLOP/s vector
                                    peak); inputs drawn on the device with the workload's distributions;
                                    --no-sweep skips it,
  cpu_baseline                      the CPU oracle timed on this machine's host cores (all threads; beside it one
                                    thread, and the oracle's exact backward).
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
MIN_LAUNCHES = 100             # medians are taken over at least this many launches
BATCH = 10                     # ... timed in batches of this many back-to-back launches


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


def sweep_cases(workloads):
    """(workload name, rank, order) of every benchmark row: the five configurations' ranks and
    orders (the tiny fp32 exactness case included), the 49-token maps, the 197-token sequences and two small batches."""
    for name, wl in workloads.WORKLOADS.items():
        for r in wl.ranks:
            for order in wl.orders:
                yield name, r, order


class Timer:
    """Event timing on torch's current stream, which is the stream every library call is given."""

    def __init__(self, torch):
        self.torch = torch

    def settle(self, step, seconds=0.05):
        """Untimed launches for `seconds`: clocks and caches reach their steady state before anything is timed."""
        t0, i = time.perf_counter(), 0
        while time.perf_counter() - t0 < seconds:
            for _ in range(10):
                step(i)
                i += 1
            self.torch.cuda.synchronize()

    def loop(self, step, steps, warmup):
        """The contract's loop: `warmup` untimed steps, then exactly `steps` between two events."""
        torch = self.torch
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            step(warmup + i)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return e0.elapsed_time(e1) / steps, wall_ms / steps

    def launches(self, step, n=MIN_LAUNCHES, warmup=10, batch=BATCH):
        """At least n launches in batches of `batch` back-to-back launches, every batch between its
        own pair of events: (median over the batches of the time per launch, mean over all launches,
        median of the same number of launches each between its own pair of events), in ms.  An event
        between two launches costs about 2 us on this machine (its packet drains the queue), which
        the third figure carries on every launch and the first on every tenth."""
        torch = self.torch
        nb = (max(n, MIN_LAUNCHES) + batch - 1) // batch
        for i in range(warmup):
            step(i)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(nb + 1)]
        torch.cuda.synchronize()
        ev[0].record()
        for b in range(nb):
            for i in range(batch):
                step(warmup + b * batch + i)
            ev[b + 1].record()
        torch.cuda.synchronize()
        t = np.array([ev[b].elapsed_time(ev[b + 1]) for b in range(nb)]) / batch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(nb * batch + 1)]
        ev[0].record()
        for i in range(nb * batch):
            step(warmup + i)
            ev[i + 1].record()
        torch.cuda.synchronize()
        single = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(nb * batch)])
        return float(np.median(t)), float(t.mean()), float(np.median(single))


class Case:
    """One (workload, rank, order) on the device: rotating buffer sets and, per set, the argument
    list of every library call the benchmark makes (built once; a launch is then one ctypes call)."""

    def __init__(self, torch, binding, workloads, wl, r, order, seeded=True, warm=False):
        self.torch, self.binding, self.wl, self.r, self.order = torch, binding, wl, r, order
        self.lib = binding.load()
        self.idx = binding.select_bases(wl.patch, r, order)
        self.seq = wl.extra > 0
        self.esz = 4 if wl.dtype == "f32" else 2
        T = wl.H * wl.W + wl.extra
        self.host = None
        if seeded:
            self.host = workloads.make_token_inputs(wl, wl.extra) if self.seq else workloads.make_inputs(wl)
            base = {k: self._to_dev(v, workloads) for k, v in self.host.items()}
        else:
            base = self._device_inputs()
        set_bytes = sum(t.numel() * t.element_size() for t in base.values()) + base["x"].numel() * self.esz \
            + base["w"].numel() * 4
        self.n_sets = 1 if warm else max(2, int(np.ceil(600e6 / set_bytes)))
        self.sets = []
        for i in range(self.n_sets):
            s = {k: (v if i == 0 else v.clone()) for k, v in base.items()}
            s["gx"] = torch.empty_like(s["x"])
            s["gW"] = torch.empty(s["w"].shape, dtype=torch.float32, device="cuda")
            self.sets.append(s)
        dt = binding.LBP_F32 if wl.dtype == "f32" else binding.LBP_BF16
        self.shape = binding.LbpShape(wl.N, wl.H, wl.W, wl.Cin, wl.Cout, dt, binding.LBP_F32)
        # the exact backward sees a token sequence as one long row of a grid
        self.full_shape = binding.LbpShape(wl.N, 1, T, wl.Cin, wl.Cout, dt, binding.LBP_F32) if self.seq else self.shape
        self.idx_arr = (ctypes.c_int32 * len(self.idx))(*self.idx)
        self.stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        Mr = wl.patches * r + wl.N * wl.extra
        tdt = base["x"].dtype
        for s in self.sets:
            s["x_r"] = torch.empty((Mr, wl.Cin), dtype=tdt, device="cuda")
            s["gy_r"] = torch.empty((Mr, wl.Cout), dtype=tdt, device="cuda")
        self.calls = {k: [self._args(k, s) for s in self.sets] for k in
                      ("lbp", "full", "full_gx", "full_gw", "pre", "proj", "prod", "prod_gw", "prod_gx")}
        # fill x_r / gy_r of every set once (the products-alone and kept-projection calls read them)
        for i in range(self.n_sets):
            self.run("proj", i)
        torch.cuda.synchronize()

    def _to_dev(self, a, workloads):
        torch = self.torch
        if self.wl.dtype == "f32":
            return torch.from_numpy(a).cuda()
        return torch.from_numpy(workloads.bf16_bits(a).reshape(a.shape).view(np.int16)).cuda().view(torch.bfloat16)

    def _device_inputs(self):
        """Inputs of the workload's distributions drawn on the device (timing rows of the sweep: the
        values only have to look like the seeded ones; nothing is compared)."""
        torch, wl = self.torch, self.wl
        gen = torch.Generator(device="cuda").manual_seed(wl.seed)
        x = torch.nn.functional.gelu(torch.randn((wl.N, wl.H, wl.W, wl.Cin), generator=gen, device="cuda"))
        w = 0.02 * torch.randn((wl.Cout, wl.Cin), generator=gen, device="cuda")
        coarse = 1e-2 * torch.randn((wl.N, wl.Cout, 4, 4), generator=gen, device="cuda")
        gy = torch.nn.functional.interpolate(coarse, size=(wl.H, wl.W), mode="bilinear", align_corners=True)
        gy = gy.permute(0, 2, 3, 1).contiguous()
        gy += 1e-3 * torch.randn(gy.shape, generator=gen, device="cuda")
        del coarse
        if self.seq:
            xe = torch.nn.functional.gelu(torch.randn((wl.N, wl.extra, wl.Cin), generator=gen, device="cuda"))
            ge = 1e-2 * torch.randn((wl.N, wl.extra, wl.Cout), generator=gen, device="cuda")
            x = torch.cat([xe, x.view(wl.N, -1, wl.Cin)], dim=1).contiguous()
            gy = torch.cat([ge, gy.view(wl.N, -1, wl.Cout)], dim=1).contiguous()
        if wl.dtype == "f32":
            return {"x": x, "gy": gy, "w": w}
        return {"x": x.to(torch.bfloat16), "gy": gy.to(torch.bfloat16), "w": w.to(torch.bfloat16)}

    def _args(self, kind, s):
        """[(C function, argument tuple), ...] of one benchmark call on buffer set s."""
        lib, wl, P = self.lib, self.wl, ctypes.c_void_p
        p = {k: P(v.data_ptr()) for k, v in s.items()}
        sh, fsh = ctypes.byref(self.shape), ctypes.byref(self.full_shape)
        idx, r, st, patch, none = self.idx_arr, self.r, self.stream, wl.patch, None
        dt = self.shape.dtype
        if kind == "lbp":
            if self.seq:
                return [(lib.lbp_wht_backward_tokens, (p["x"], p["gy"], p["w"], sh, wl.extra, patch, idx, r, p["gx"], p["gW"], st))]
            return [(lib.lbp_wht_backward, (p["x"], p["gy"], p["w"], sh, patch, idx, r, p["gx"], p["gW"], st))]
        if kind == "full":
            return [(lib.full_bp_backward, (p["x"], p["gy"], p["w"], fsh, p["gx"], p["gW"], st))]
        if kind == "full_gx":
            return [(lib.full_bp_backward, (p["x"], p["gy"], p["w"], fsh, p["gx"], none, st))]
        if kind == "full_gw":
            return [(lib.full_bp_backward, (p["x"], p["gy"], p["w"], fsh, none, p["gW"], st))]
        if kind == "pre":
            if self.seq:
                return [(lib.lbp_wht_backward_tokens_preprojected,
                         (p["x_r"], p["gy"], p["w"], sh, wl.extra, patch, idx, r, p["gx"], p["gW"], st))]
            return [(lib.lbp_wht_backward_preprojected, (p["x_r"], p["gy"], p["w"], sh, patch, idx, r, p["gx"], p["gW"], st))]
        if kind == "proj":
            return [(lib.lbp_wht_project_pair_tokens, (p["x"], p["gy"], sh, wl.extra, patch, idx, r, p["x_r"], p["gy_r"], st))]
        gx, gW = (none if kind == "prod_gw" else p["gx"]), (none if kind == "prod_gx" else p["gW"])
        return [(lib.lbp_wht_products_tokens, (p["x_r"], p["gy_r"], p["w"], sh, wl.extra, patch, idx, r, gx, gW, st))]

    def run(self, kind, i):
        for fn, a in self.calls[kind][i % self.n_sets]:
            rc = fn(*a)
            if rc != 0:
                raise self.binding.LbpError(rc, self.binding.strerror(rc), self.lib.lbp_last_hip_error())

    def step(self, kind):
        return lambda i: self.run(kind, i)

    # ---- algorithmic work of the two kernels the roofline is about
    @property
    def Mr(self):
        return self.wl.patches * self.r + self.wl.N * self.wl.extra

    def proj_bytes(self):
        """Projection launch: read gy and x once, write the r/p^2 fraction of each (and the tokens
        outside the grid as they are)."""
        wl = self.wl
        return self.esz * (wl.tokens + self.Mr) * (wl.Cout + wl.Cin)

    def products_flops(self):
        """Both products: 2 * M_r * Cin * Cout each."""
        return 4.0 * self.Mr * self.wl.Cin * self.wl.Cout

    def products_bytes(self):
        wl = self.wl
        return self.esz * (self.Mr * (wl.Cin + wl.Cout) + wl.Cin * wl.Cout + wl.tokens * wl.Cin) + 4 * wl.Cin * wl.Cout

    def plan_text(self):
        return self.binding.describe_plan(self.shape, self.wl.patch, self.idx, extra=self.wl.extra)


def sweep_row(case, timer, full_us):
    """One row of the per-(configuration, rank, order) table; times are medians of >= 100 launches."""
    wl = case.wl
    lbp = timer.launches(case.step("lbp"))[0] * 1e3
    proj = timer.launches(case.step("proj"))[0] * 1e3
    peak = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else 157.3      # fp32 products run on the vector units
    row = {"workload": wl.name, "dtype": wl.dtype, "r": case.r, "order": case.order, "lbp_us": round(lbp, 1),
           "full_bp_us": round(full_us, 1), "speedup": round(full_us / lbp, 2), "proj_us": round(proj, 1),
           "proj_frac_hbm": round(case.proj_bytes() / (proj * 1e-6) / 1e9 / HBM_PEAK_GBS, 3),
           "prod_us": None, "prod_frac_peak": None}
    prod = timer.launches(case.step("prod"))[0] * 1e3
    row["prod_us"] = round(prod, 1)
    row["prod_frac_peak"] = round(case.products_flops() / (prod * 1e-6) / 1e12 / peak, 3)
    return row


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
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-(configuration, rank, order) table")
    ap.add_argument("--sweep-table", default=None, help="also write the sweep as a text table to this file")
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
    timer = Timer(torch)
    wl = workloads.WORKLOADS[args.workload]
    r = args.rank or wl.ranks[0]
    case = Case(torch, binding, workloads, wl, r, args.order, seeded=True, warm=args.warm_cache)
    seq, n_sets, sets, idx = case.seq, case.n_sets, case.sets, case.idx

    # medians first, then the contract's loop of exactly --steps steps
    timer.settle(case.step("lbp"))
    med_lbp, mean_lbp, b2b_lbp = timer.launches(case.step("lbp"))
    ms_lbp, wall_lbp = timer.loop(case.step("lbp"), args.steps, args.warmup)
    # the cache-warm number beside it, labelled: one buffer set over and over
    ms_warm = None if args.warm_cache else timer.launches(lambda i: case.run("lbp", 0))[0]
    # the same steps recorded once into a HIP graph (one step per buffer set) and replayed: what a
    # training loop that captures its backward pass sees; launch gaps between the kernels shrink
    ms_graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):      # capture runs on a stream of its own: the binding passes the current one
            for s in sets:
                if seq:
                    binding.lbp_wht_backward_tokens(s["x"], s["gy"], s["w"], (wl.H, wl.W), wl.patch, idx, gx=s["gx"], gW=s["gW"])
                else:
                    binding.lbp_wht_backward(s["x"], s["gy"], s["w"], wl.patch, idx, gx=s["gx"], gW=s["gW"])
        ms_graph = timer.launches(lambda i: graph.replay(), 30, batch=1)[0] / n_sets
    # the variant that keeps x^ from the forward pass (never reads x)
    ms_pre = timer.launches(case.step("pre"))[0]
    # the two kernels of a call, each by itself on the launch stream (same rotation of buffers)
    med_proj, mean_proj, b2b_proj = timer.launches(case.step("proj"))
    med_prod, mean_prod, b2b_prod = timer.launches(case.step("prod"))
    ms_full = timer.launches(case.step("full"))[0]
    ms_lib = ms_lib_lowrank = ms_best_full = full_parts = None
    if not args.no_library_gemm:
        def lib_step(i):
            s = sets[i % n_sets]
            G = s["gy"].view(-1, wl.Cout)
            torch.matmul(G, s["w"], out=s["gx"].view(-1, wl.Cin))
            torch.matmul(G.t(), s["x"].view(-1, wl.Cin))      # allocates its result: the library's habit, not timed apart

        def lib_gx(i):
            s = sets[i % n_sets]
            torch.matmul(s["gy"].view(-1, wl.Cout), s["w"], out=s["gx"].view(-1, wl.Cin))

        def lib_gw(i):
            s = sets[i % n_sets]
            torch.matmul(s["gy"].view(-1, wl.Cout).t(), s["x"].view(-1, wl.Cin))

        ms_lib = timer.launches(lib_step)[0]
        # the strongest exact backward on hand: each of its two products from whichever of this
        # library and the vendor's is faster, each timed alone
        full_parts = {"own_gx_ms": timer.launches(case.step("full_gx"))[0], "own_gw_ms": timer.launches(case.step("full_gw"))[0],
                      "library_gx_ms": timer.launches(lib_gx)[0], "library_gw_ms": timer.launches(lib_gw)[0]}
        ms_best_full = min(full_parts["own_gx_ms"], full_parts["library_gx_ms"]) + \
            min(full_parts["own_gw_ms"], full_parts["library_gw_ms"])
        # the two LOW-RANK products through the vendor GEMM library, from the projected tensors
        # (no reverse projection, no 1/p^2): what a library call costs on shapes this small
        lr_out = [torch.empty((case.Mr, wl.Cin), dtype=s["x_r"].dtype, device="cuda") for s in sets]

        def lib_lowrank_step(i):
            s = sets[i % n_sets]
            torch.matmul(s["gy_r"], s["w"], out=lr_out[i % n_sets])
            torch.matmul(s["gy_r"].t(), s["x_r"])

        ms_lib_lowrank = timer.launches(lib_lowrank_step)[0]

    # where the time of a call goes: the two products launched alone
    ms_gw = timer.launches(case.step("prod_gw"))[0]
    ms_gx = timer.launches(case.step("prod_gx"))[0]

    if args.calibration_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()

    flops = lbp_flops(wl, r)
    proj_bytes = case.proj_bytes()
    proj_gbs = proj_bytes / (med_proj * 1e-3) / 1e9
    traffic_file = f"wht_project_{wl.name}_hbm_traffic.txt"
    roof_proj = {"bound": "hbm", "kernel": "projection of gy and x (one launch)",
                 "achieved": round(proj_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": round(proj_gbs / HBM_PEAK_GBS, 4),
                 "traffic": read_traffic(traffic_file, r, args.order),
                 "traffic_source": f"profiles/{traffic_file} (stored rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE reading, not measured in this run)",
                 "algorithmic_bytes": proj_bytes, "avg_launch_us": round(med_proj * 1e3, 2),
                 "mean_launch_us": round(mean_proj * 1e3, 2), "single_launch_us": round(b2b_proj * 1e3, 2),
                 "launches": MIN_LAUNCHES}
    gemm_flops = case.products_flops() / 2
    plan_products = case.plan_text().split("products: ", 1)[-1].split("; workspace", 1)[0]
    # the two products (one grouped launch where the planner groups them; with the reverse projection
    # in the epilogue where it can be fused): 2 * M_r * Cin * Cout FLOPs each against the dense bf16
    # (fp32: vector fp32) peak; launched from projected tensors
    peak = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else 157.3
    tf = 2.0 * gemm_flops / (med_prod * 1e-3) / 1e12
    traffic_file = f"gemm_products_{wl.name}_hbm_traffic.txt"
    roof_prod = {"bound": "mfma" if wl.dtype == "bf16" else "alu",
                 "kernel": "the two products of a call, g^y W with the reverse projection of Eq. 7 and g^y^T x^ (" + plan_products + ")",
                 "achieved": round(tf, 1), "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4),
                 "traffic": read_traffic(traffic_file, r, args.order),
                 "traffic_source": f"profiles/{traffic_file} (stored rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE reading, not measured in this run)",
                 "algorithmic_flops": 2.0 * gemm_flops, "avg_launch_us": round(med_prod * 1e3, 2),
                 "mean_launch_us": round(mean_prod * 1e3, 2), "single_launch_us": round(b2b_prod * 1e3, 2),
                 "launches": MIN_LAUNCHES}
    # the other candidate bound: operands read once, outputs written once
    prod_bytes = case.products_bytes()
    roof_prod["algorithmic_bytes"] = prod_bytes
    roof_prod["frac_of_hbm_peak"] = round(prod_bytes / (med_prod * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    # `roofline` is the kernel that takes the larger share of a step, `roofline_second` the other
    if med_prod > med_proj:
        roofline, roofline_second = roof_prod, roof_proj
    else:
        roofline, roofline_second = roof_proj, roof_prod
    stages = {
        "projection_us": round(med_proj * 1e3, 2),
        "products_us": round(med_prod * 1e3, 2),
        "gw_product_alone_us": round(ms_gw * 1e3, 2),
        "gx_product_reverse_projection_alone_us": round(ms_gx * 1e3, 2),
        "gw_product_alone_frac_of_mfma_peak": round(gemm_flops / (ms_gw * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "gx_product_alone_frac_of_mfma_peak": round(gemm_flops / (ms_gx * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
    }

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        host, grid = case.host, (wl.H, wl.W)
        # bounded sample: as many leading images as keep the oracle's work near 20 GFLOP
        n_s = int(max(1, min(wl.N, round(wl.N * 20e9 / max(flops, 1.0)))))
        sample = {k: (v[:n_s] if k != "w" else v) for k, v in host.items()}
        wl_s = workloads.scaled(wl, N=n_s)
        best = 1e30
        for _ in range(5):
            t0 = time.perf_counter()
            if seq:
                oracle.lbp_wht_backward_tokens(sample["x"], sample["gy"], sample["w"], grid, wl.patch, np.asarray(idx))
            else:
                oracle.lbp_wht_backward_padded(sample["x"], sample["gy"], sample["w"], wl.patch, np.asarray(idx))
            best = min(best, time.perf_counter() - t0)
        threads = oracle.max_threads()
        cpu = {"value": round(lbp_flops(wl_s, r) / best / 1e12, 6), "unit": "TFLOP/s",
               "cores": threads, "kind": "oracle",
               "sample": f"first {n_s} of {wl.N} images of the same workload, best of 5 calls, {best:.2f} s each",
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

    config = {"workload": wl.name, "N": wl.N, "grid": [wl.H, wl.W], "extra_tokens": wl.extra, "Cin": wl.Cin,
              "Cout": wl.Cout, "patch": wl.patch, "r": r, "order": args.order,
              "cache": "warm" if args.warm_cache else f"cold ({n_sets} rotating buffer sets)"}

    # the table the benchmark spec asks for: every configuration, rank and order
    sweep = None
    if not args.no_sweep:
        del case, sets
        torch.cuda.empty_cache()
        sweep, full_us, last = [], {}, None
        for name, rr, order in sweep_cases(workloads):
            w2 = workloads.WORKLOADS[name]
            c = Case(torch, binding, workloads, w2, rr, order, seeded=False)
            timer.settle(c.step("lbp"))       # allocating and filling the case's tensors let the clocks drop
            if name not in full_us:
                full_us[name] = timer.launches(c.step("full"))[0] * 1e3
            sweep.append(sweep_row(c, timer, full_us[name]))
            del c
            if last != name:
                torch.cuda.empty_cache()
                last = name
        if args.sweep_table:
            with open(args.sweep_table, "w") as f:
                f.write(f"{'workload':22s} {'r':>3s} {'order':>5s} {'lbp_us':>8s} {'full_us':>8s} {'speedup':>7s} "
                        f"{'proj_us':>7s} {'hbm':>5s} {'prod_us':>7s} {'peak':>5s}\n")
                for row in sweep:
                    pu = "-" if row["prod_us"] is None else f"{row['prod_us']:.1f}"
                    pf = "-" if row["prod_frac_peak"] is None else f"{row['prod_frac_peak']:.3f}"
                    f.write(f"{row['workload']:22s} {row['r']:3d} {row['order']:>5s} {row['lbp_us']:8.1f} {row['full_bp_us']:8.1f} "
                            f"{row['speedup']:7.2f} {row['proj_us']:7.1f} {row['proj_frac_hbm']:5.3f} {pu:>7s} {pf:>5s}\n")

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
        "config": config,
        "timing": f"ms_per_step: exactly --steps steps between two events after --warmup steps; every other figure: median over "
                  f"{MIN_LAUNCHES // BATCH} batches of {BATCH} back-to-back launches, each batch between its own pair of events",
        "ms_per_step_median": round(med_lbp, 5),
        "ms_per_step_single_launches": round(b2b_lbp, 5),
        "lbp_flops_per_step": flops,
        "bp_equivalent_tflops": round(full_bp_flops(wl) / (ms_lbp * 1e-3) / 1e12, 3),
        "full_bp_ms": round(ms_full, 5),
        "full_bp_tflops": round(full_bp_flops(wl) / (ms_full * 1e-3) / 1e12, 3),
        "speedup_vs_full_bp": round(ms_full / ms_lbp, 3),
        "library_gemm_full_bp_ms": None if ms_lib is None else round(ms_lib, 5),
        "speedup_vs_library_gemm_full_bp": None if ms_lib is None else round(ms_lib / ms_lbp, 3),
        "best_of_both_full_bp_ms": None if ms_best_full is None else round(ms_best_full, 5),
        "speedup_vs_best_of_both_full_bp": None if ms_best_full is None else round(ms_best_full / ms_lbp, 3),
        "full_bp_products_alone_ms": None if full_parts is None else {k: round(v, 5) for k, v in full_parts.items()},
        "library_gemm_lowrank_products_ms": None if ms_lib_lowrank is None else round(ms_lib_lowrank, 5),
        "preprojected_x_ms_per_step": round(ms_pre, 5),
        "preprojected_x_speedup_vs_full_bp": round(ms_full / ms_pre, 3),
        "graph_replay_ms_per_step": None if ms_graph is None else round(ms_graph, 5),
        "host_wall_ms_per_step": round(wall_lbp, 5),
        "warm_cache_ms_per_step": None if ms_warm is None else round(ms_warm, 5),
        "stages": stages,
        "roofline": roofline,
        "roofline_second": roofline_second,
        "sweep": sweep,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
