"""Seeded random shapes through the whole backward call: grids that are and are not multiples of
the patch, channel counts with ragged tiles, low-pass and arbitrary basis lists, both dtypes,
default kernel choices.  Every case is compared element by element with the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from _gpu_util import TOL, assert_matches, device_inputs, full_backward, lbp_backward
from paper_2309_15275_amd import binding
from paper_2309_15275_amd.workloads import Workload

pytestmark = pytest.mark.gpu

N_CASES = 48


def draw_case(i):
    rng = np.random.default_rng(7000 + i)
    dtype = "bf16" if i % 3 else "f32"
    patch = int(rng.choice([2, 4, 8, 8, 8, 16]))
    vec = 8 if dtype == "bf16" else 4
    N = int(rng.integers(1, 5))
    if rng.random() < 0.5:
        H, W = int(rng.integers(1, 4)) * patch, int(rng.integers(1, 4)) * patch
    else:
        H, W = int(rng.integers(1, 3 * patch + 1)), int(rng.integers(1, 3 * patch + 1))
    Cin, Cout = int(rng.integers(1, 40)) * vec, int(rng.integers(1, 40)) * vec
    pp = patch * patch
    kind = int(rng.integers(0, 3))
    if kind == 0:
        r = int(rng.integers(1, min(pp, 40) + 1))
        idx = oracle.select_bases(patch, r, "l1" if rng.random() < 0.5 else "linf")
    elif kind == 1:
        r = int(rng.integers(1, min(pp, 24) + 1))
        idx = rng.permutation(pp)[:r].astype(np.int32)          # arbitrary and unordered, as LHE could return
    else:
        k = int(rng.integers(1, min(patch, 4) + 1))             # a whole LP_Linf square: poolable
        idx = oracle.select_bases(patch, k * k, "linf")
    return Workload(f"random{i}", N, H, W, Cin, Cout, patch, (), ("l1",), dtype, 9000 + i), np.asarray(idx)


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_case_matches_the_oracle(i):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    wl, idx = draw_case(i)
    print(f"case {i}: N={wl.N} grid={wl.H}x{wl.W} Cin={wl.Cin} Cout={wl.Cout} patch={wl.patch} dtype={wl.dtype} idx={idx.tolist()}",
          flush=True)
    host, dev = device_inputs(wl)
    gx, gW = lbp_backward(dev, wl.patch, idx)
    gx0, gW0 = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], wl.patch, idx)
    assert_matches(gx, gx0, TOL[wl.dtype], "gx")
    assert_matches(gW, gW0, TOL[wl.dtype], "gW")


N_BIG = 40


def draw_big_case(i):
    """Larger layers (up to 1536 channels, up to 16 images): many GEMM tiles per product, so that the
    tile-to-XCD numbering, split-K and the grouped launch see shapes the benchmark configurations do not."""
    rng = np.random.default_rng(9100 + i)
    patch = int(rng.choice([4, 8, 8, 8]))
    N = int(rng.integers(1, 17))
    H, W = int(rng.integers(1, 5)) * patch - int(rng.integers(0, 2)), int(rng.integers(1, 5)) * patch
    Cin, Cout = int(rng.integers(8, 193)) * 8, int(rng.integers(8, 193)) * 8
    pp = patch * patch
    r = int(rng.choice([1, 3, 4, 8, 10, 15, 16, 21, 36])) if patch == 8 else int(rng.integers(1, pp + 1))
    idx = oracle.select_bases(patch, min(r, pp), "l1" if rng.random() < 0.6 else "linf")
    return Workload(f"big{i}", N, H, W, Cin, Cout, patch, (), ("l1",), "bf16", 9500 + i), np.asarray(idx)


@pytest.mark.parametrize("i", range(N_BIG))
def test_larger_random_case_matches_the_oracle(i):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    wl, idx = draw_big_case(i)
    print(f"big case {i}: N={wl.N} grid={wl.H}x{wl.W} Cin={wl.Cin} Cout={wl.Cout} patch={wl.patch} r={len(idx)}", flush=True)
    host, dev = device_inputs(wl)
    gx, gW = lbp_backward(dev, wl.patch, idx)
    gx0, gW0 = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], wl.patch, idx)
    assert_matches(gx, gx0, TOL["bf16"], "gx")
    assert_matches(gW, gW0, TOL["bf16"], "gW")
    if i % 3 == 0:
        fx, fW = full_backward(dev)
        f0, w0 = oracle.full_bp_backward(host["x"], host["gy"], host["w"])
        assert_matches(fx, f0, 5e-3, "exact gx")
        assert_matches(fW, w0, 5e-3, "exact gW")
