"""The entry point that allocates nothing (lbp_wht_backward_static): through the C ABI, against
lbp_wht_backward on the same inputs, two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle
from _gpu_util import TOL, assert_matches, device_inputs, nan_outputs
from paper_2309_15275_amd import binding
from paper_2309_15275_amd.workloads import Workload

pytestmark = pytest.mark.gpu


def _case(N, H, W, Cin, Cout, patch, r, seed):
    wl = Workload("static", N, H, W, Cin, Cout, patch, (), ("l1",), "bf16", seed)
    host, dev = device_inputs(wl)
    return wl, host, dev, oracle.select_bases(patch, r, "l1")


def test_static_scratch_backward_two_calls_the_second_smaller():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    # first: the weight gradient leaves split-K partial sums in the scratch array (besides the projected
    # tensors); second: split-K slices of unfused input-gradient coefficients; last: a smaller, fused call
    cases = [_case(6, 16, 32, 264, 520, 8, 21, 811), _case(4, 16, 16, 136, 4096, 8, 21, 813),
             _case(2, 16, 16, 72, 136, 8, 8, 812)]
    for wl, host, dev, idx in cases:
        print(f"static call N={wl.N} grid={wl.H}x{wl.W} {wl.Cin}->{wl.Cout} r={len(idx)}: "
              + binding.describe_plan(binding.make_shape(dev["x"], dev["gy"], dev["w"]), wl.patch, idx), flush=True)
        gx, gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape)
        binding.lbp_wht_backward_static(dev["x"], dev["gy"], dev["w"], wl.patch, idx, gx, gW)
        ref_gx, ref_gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape)
        binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx, gx=ref_gx, gW=ref_gW)
        torch.cuda.synchronize()
        # the same kernels on the same plan: the same bits
        assert torch.equal(gx.view(torch.int16), ref_gx.view(torch.int16))
        assert torch.equal(gW.view(torch.int32), ref_gW.view(torch.int32))
        gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], wl.patch, idx)
        assert_matches(gx, gx0, TOL["bf16"], "gx")
        assert_matches(gW, gW0, TOL["bf16"], "gW")


def test_static_scratch_backward_rejects_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    # 128 images of 32 x 32 tokens, 768 channels, all 64 bases: the projected tensors alone are 2 x 201 MB
    N, H, W, C = 128, 32, 32, 768
    x = torch.zeros((N, H, W, C), dtype=torch.bfloat16, device="cuda")
    gy = torch.zeros((N, H, W, C), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((C, C), dtype=torch.bfloat16, device="cuda")
    gx = torch.full_like(x, 3.0)
    gW = torch.full((C, C), 3.0, dtype=torch.float32, device="cuda")
    shape = binding.make_shape(x, gy, w)
    assert binding.workspace_bytes(shape, 8, 64) > binding.STATIC_SCRATCH_BYTES
    with pytest.raises(binding.LbpError) as e:
        binding.lbp_wht_backward_static(x, gy, w, 8, np.arange(64), gx, gW)
    assert e.value.code == -10
    torch.cuda.synchronize()
    assert bool((gx == 3.0).all()) and bool((gW == 3.0).all())      # nothing was launched


def test_static_scratch_backward_inside_a_captured_graph():
    # what the entry point is for: a caller under graph capture.  After one eager call (kernel attributes
    # set) the call is recorded and replayed with new inputs in the same buffers; every replay must
    # reproduce the eager lbp_wht_backward bit for bit.
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    wl, host, dev, idx = _case(4, 16, 16, 136, 264, 8, 8, 815)
    gx, gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape)
    binding.lbp_wht_backward_static(dev["x"], dev["gy"], dev["w"], wl.patch, idx, gx, gW)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.lbp_wht_backward_static(dev["x"], dev["gy"], dev["w"], wl.patch, idx, gx, gW)
    for rep in range(3):
        with torch.no_grad():
            dev["gy"].mul_(-0.5 if rep % 2 else 2.0)           # exact in bf16: new inputs, same buffers
            dev["x"].copy_(dev["x"].roll(1, dims=0))
        gx.fill_(float("nan"))
        gW.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        ref_gx, ref_gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
        torch.cuda.synchronize()
        assert torch.equal(gx, ref_gx) and torch.equal(gW, ref_gW), rep


def test_static_scratch_backward_with_a_reduction_cut_inside_the_launch_under_a_graph():
    # the input-gradient product's reduction in 3 slices that join inside the launch: partial tiles in the scratch
    # array, tile counters in the library's device image, nothing allocated; replays start from clean counters
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.set_option("LBP_GX_JOIN", "3")
    try:
        wl, host, dev, idx = _case(2, 16, 16, 136, 776, 8, 8, 817)
        text = binding.describe_plan(binding.make_shape(dev["x"], dev["gy"], dev["w"]), wl.patch, idx)
        assert "reduction in 3 slices joined in the launch" in text, text
        gx, gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape)
        binding.lbp_wht_backward_static(dev["x"], dev["gy"], dev["w"], wl.patch, idx, gx, gW)
        torch.cuda.synchronize()
        gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], wl.patch, idx)
        assert_matches(gx, gx0, TOL["bf16"], "gx")
        assert_matches(gW, gW0, TOL["bf16"], "gW")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            binding.lbp_wht_backward_static(dev["x"], dev["gy"], dev["w"], wl.patch, idx, gx, gW)
        for rep in range(3):
            with torch.no_grad():
                dev["gy"].mul_(-0.5 if rep % 2 else 2.0)
                dev["x"].copy_(dev["x"].roll(1, dims=0))
            gx.fill_(float("nan"))
            gW.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            ref_gx, ref_gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
            torch.cuda.synchronize()
            assert torch.equal(gx, ref_gx) and torch.equal(gW, ref_gW), rep
    finally:
        binding.reset_options()
