"""Runs bench.py once per benchmark configuration, rank and basis order and prints one table:
time of the LBP-WHT backward, of the full-rank backward built from the same kernels, of the same
two products through the vendor GEMM library, the speedups, the three stage times and the
achieved bandwidth of the projection launch.

    python -m paper_2309_15275_amd.sweep [--steps 100] [--warmup 20] [--out table.txt]

Every row is a fresh `python bench.py --no-cpu-baseline ...` process (one GPU)."""
import argparse
import json
import os
import subprocess
import sys

from . import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def cases():
    for name, wl in workloads.WORKLOADS.items():
        for r in wl.ranks:
            for order in wl.orders:
                yield name, r, order


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    head = (f"{'workload':22s} {'r':>3s} {'order':>5s} {'lbp_us':>8s} {'full_us':>8s} {'lib_us':>8s} {'speedup':>7s} "
            f"{'vs_lib':>6s} {'pre_us':>7s} {'proj':>6s} {'prods':>6s} {'gW':>6s} {'gx':>6s} {'proj GB/s':>9s} {'frac':>5s}")
    lines = [head]
    print(head, flush=True)
    for name, r, order in cases():
        cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--no-cpu-baseline", "--steps", str(args.steps),
               "--warmup", str(args.warmup), "--workload", name, "--rank", str(r), "--order", order]
        res = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT, timeout=600)
        if res.returncode != 0:
            line = f"{name:22s} {r:3d} {order:>5s} FAILED (exit {res.returncode})"
        else:
            j = json.loads(res.stdout.strip().splitlines()[-1])
            ro = j["roofline"] if j["roofline"]["bound"] == "hbm" else j["roofline_second"]      # the projection launch
            nan = float("nan")
            st = j["stages"] or {"projection_us": nan, "products_us": nan, "gw_product_alone_us": nan,
                                 "gx_product_reverse_projection_alone_us": nan}      # none for token sequences
            lib = j["library_gemm_full_bp_ms"]
            line = (f"{name:22s} {r:3d} {order:>5s} {j['ms_per_step'] * 1e3:8.1f} {j['full_bp_ms'] * 1e3:8.1f} "
                    f"{lib * 1e3:8.1f} {j['speedup_vs_full_bp']:7.2f} {j['speedup_vs_library_gemm_full_bp']:6.2f} "
                    f"{j['preprojected_x_ms_per_step'] * 1e3:7.1f} {st['projection_us']:6.1f} {st['products_us']:6.1f} "
                    f"{st['gw_product_alone_us']:6.1f} {st['gx_product_reverse_projection_alone_us']:6.1f} "
                    f"{ro['achieved']:9.0f} {ro['frac']:5.2f}")
        lines.append(line)
        print(line, flush=True)
    if args.out:
        with open(args.out, "w") as f:
            f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
