"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (default paths, planner-chosen tiles).  Every configuration, rank and order is
compared with the whole oracle element by element (norm, every row, every element; outputs start
as NaN); only the tensors beyond 2^31 elements are compared on sampled patches, rows and entries
that the oracle computes one by one."""
import os

import numpy as np
import pytest
import torch

import oracle
from _gpu_util import TOL, assert_matches, device_inputs, full_backward, lbp_backward, rel_fro, to_host
from paper_2309_15275_amd import binding, workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    yield
    binding.reset_options()
    torch.cuda.synchronize()


def check_whole(wl, host, gx, gW, idx):
    """gx and gW of a call against Algorithm 1 on the whole tensors (zero-padded grids included)."""
    fn = oracle.lbp_wht_backward_padded if (wl.H % wl.patch or wl.W % wl.patch) else oracle.lbp_wht_backward
    gx0, gW0 = fn(host["x"], host["gy"], host["w"], wl.patch, idx)
    return assert_matches(gx, gx0, TOL[wl.dtype], "gx"), assert_matches(gW, gW0, TOL[wl.dtype], "gW")


def test_cfg2_vitb_fc1_whole_oracle():
    wl = workloads.WORKLOADS["cfg2_vitb_fc1"]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, 8, "l1")
    gx, gW = lbp_backward(dev, wl.patch, idx)
    check_whole(wl, host, gx, gW, idx)


def test_cfg2_full_rank_backward_whole_oracle():
    wl = workloads.WORKLOADS["cfg2_vitb_fc1"]
    host, dev = device_inputs(wl)
    gx, gW = full_backward(dev)
    gx0, gW0 = oracle.full_bp_backward(host["x"], host["gy"], host["w"])
    assert_matches(gx, gx0, 5e-3, "exact gx")
    assert_matches(gW, gW0, 5e-3, "exact gW")


def test_cfg3_thin_channels_whole_oracle():
    wl = workloads.WORKLOADS["cfg3_effformer_early"]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, 8, "l1")
    gx, gW = lbp_backward(dev, wl.patch, idx)
    check_whole(wl, host, gx, gW, idx)


@pytest.mark.parametrize("r", [8, 36])
def test_49_token_maps_whole_oracle(r):
    # 7 x 7 grids inside one zero-padded 8 x 8 patch each, at the channel counts of Section 3.3's example
    wl = workloads.WORKLOADS["pad_7x7_fc2"]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, r, "l1")
    gx, gW = lbp_backward(dev, wl.patch, idx)
    check_whole(wl, host, gx, gW, idx)


@pytest.mark.parametrize("layer", ["cfg4_vitl_fc1", "cfg4_vitl_fc2"])
def test_cfg4_vitl_rank_sweep(layer):
    wl = workloads.WORKLOADS[layer]
    host, dev = device_inputs(wl)
    for r in wl.ranks:
        print(f"{layer} r={r}", flush=True)
        idx = oracle.select_bases(wl.patch, r, "l1")
        gx, gW = lbp_backward(dev, wl.patch, idx)
        check_whole(wl, host, gx, gW, idx)


def test_cfg5_the_two_orders_pick_the_same_set_except_at_16():
    for r in (4, 8, 64):
        assert sorted(binding.select_bases(8, r, "l1")) == sorted(binding.select_bases(8, r, "linf"))
    assert sorted(binding.select_bases(8, 16, "l1")) != sorted(binding.select_bases(8, 16, "linf"))


@pytest.mark.parametrize("r,order", [(4, "l1"), (4, "linf"), (8, "l1"), (8, "linf"), (16, "l1"), (16, "linf"),
                                     (64, "l1"), (64, "linf")])
def test_cfg5_attnproj_orders_and_ranks_whole_oracle(r, order):
    wl = workloads.WORKLOADS["cfg5_vitb_attnproj"]
    host, dev = device_inputs(wl)
    idx = np.asarray(binding.select_bases(wl.patch, r, order))
    assert np.array_equal(idx, oracle.select_bases(wl.patch, r, order))
    gx, gW = lbp_backward(dev, wl.patch, idx)
    print(f"cfg5 r={r} {order}: oracle", flush=True)
    gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], wl.patch, idx)
    assert_matches(gx, gx0, TOL["bf16"], "gx")
    assert_matches(gW, gW0, TOL["bf16"], "gW")
    if r == 64 and order == "l1":
        # all bases kept: the result is exact backpropagation (Eq. 2), and so is the oracle's
        fx, fW = oracle.full_bp_backward(host["x"], host["gy"], host["w"])
        assert_matches(gx, fx, TOL["bf16"], "gx against exact backprop")
        assert_matches(gW, fW, TOL["bf16"], "gW against exact backprop")
        del fx, fW
        gxf, gWf = full_backward(dev)
        assert_matches(gWf, gW0, 5e-3, "exact gW")
        assert_matches(gxf, gx0, 5e-3, "exact gx")


def test_rank_one_is_pool_matmul_upsample_at_full_size():
    # property that holds at any size: r = 1 (the constant basis) gives gx constant inside every patch
    wl = workloads.WORKLOADS["cfg2_vitb_fc1"]
    host, dev = device_inputs(wl)
    gx = torch.full_like(dev["x"], float("nan"))
    binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, [0], gx=gx, want_gw=False)
    assert bool(torch.isfinite(gx).all())
    g = gx.reshape(wl.N, wl.H // 8, 8, wl.W // 8, 8, wl.Cin)
    first = g[:, :, :1, :, :1, :]
    assert torch.equal(g, first.expand_as(g))


# (workload, r, order): the planner runs both products of these in one launch, with, in turn, the
# pooled fused epilogue, the matrix-core fused epilogue, few input-gradient tiles beside many
# weight-gradient tiles, a split weight-gradient product, zero-padded maps, and a thin layer.
GROUPED = [("cfg2_vitb_fc1", 8, "l1"), ("cfg2_vitb_fc1", 15, "l1"), ("cfg4_vitl_fc1", 4, "l1"),
           ("cfg4_vitl_fc1", 16, "l1"), ("cfg5_vitb_attnproj", 4, "l1"), ("pad_7x7_fc2", 8, "l1"),
           ("cfg3_effformer_early", 8, "l1")]


@pytest.mark.parametrize("case", range(len(GROUPED)))
def test_grouped_and_separate_launches_of_the_products_agree(case):
    # the planner may give the two modes different tiles, so the comparison between them is by
    # norm (bit equality under equal tiles is tested on the small shapes); both must match the oracle
    name, r, order = GROUPED[case]
    wl = workloads.WORKLOADS[name]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, r, order)
    binding.set_option("LBP_GEMM_GROUP", "0")
    gx0, gW0 = lbp_backward(dev, wl.patch, idx)
    binding.set_option("LBP_GEMM_GROUP", None)
    gx1, gW1 = lbp_backward(dev, wl.patch, idx)
    assert rel_fro(to_host(gx1), to_host(gx0)) <= TOL["bf16"] and rel_fro(to_host(gW1), to_host(gW0)) <= 1e-5
    fn = oracle.lbp_wht_backward_padded if (wl.H % wl.patch or wl.W % wl.patch) else oracle.lbp_wht_backward
    gxo, gWo = fn(host["x"], host["gy"], host["w"], wl.patch, idx)
    for gx, gW in ((gx0, gW0), (gx1, gW1)):
        assert_matches(gx, gxo, TOL["bf16"], "gx")
        assert_matches(gW, gWo, TOL["bf16"], "gW")


@pytest.mark.parametrize("path", ["auto", "mfma"])
def test_tensors_beyond_two_to_the_31_elements(path):
    # 2^19 tokens x 4352 channels = 2.28e9 bf16 elements (4.6 GB): element offsets no longer fit 31 bits.
    # The tensor is made on the device (seeded); patches sampled from its whole extent, the last
    # one included, are checked against the oracle's projection of the same values; then the
    # reverse projection of those coefficients, again against the oracle on sampled patches.
    binding.set_option("LBP_WHT_PATH", path)
    N, H, W, C, p = 512, 32, 32, 4352, 8
    gen = torch.Generator(device="cuda").manual_seed(4242)
    t = torch.randn((N, H, W, C), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    idx = oracle.select_bases(p, 4, "l1")
    coef = binding.wht_project(t, p, idx)
    Q, PW = N * (H // p) * (W // p), W // p
    rng = np.random.default_rng(7)
    qs = np.unique(np.concatenate([[0, Q - 1, Q // 2], rng.integers(0, Q, 24)]))
    for q in qs:
        n, rem = divmod(int(q), (H // p) * PW)
        a, b = divmod(rem, PW)
        patch = t[n, a * p:(a + 1) * p, b * p:(b + 1) * p, :].float().cpu().numpy()[None]       # [1, p, p, C]
        want = oracle.project(patch, p, idx)                                                   # [4, C]
        got = to_host(coef[q * 4:(q + 1) * 4])
        assert rel_fro(got, want) <= 4e-3, (int(q), rel_fro(got, want))
    del t
    # reverse direction at the same size: fp32 coefficients -> bf16 tokens
    back = binding.wht_unproject(coef.float(), (N, H, W, C), torch.bfloat16, p, idx)
    for q in qs[-6:]:
        n, rem = divmod(int(q), (H // p) * PW)
        a, b = divmod(rem, PW)
        c = to_host(coef[q * 4:(q + 1) * 4])
        want = oracle.unproject(c, (1, p, p, C), p, idx)
        got = to_host(back[n, a * p:(a + 1) * p, b * p:(b + 1) * p, :])[None]
        assert rel_fro(got, want) <= 4e-3, int(q)
    binding.set_option("LBP_WHT_PATH", None)


def test_backward_with_more_than_two_to_the_31_input_elements():
    # x and gx have 2^19 tokens x 4352 channels (2.28e9 elements); gy is narrow.  Sampled rows of gx
    # (the last token included) and sampled entries of gW against the oracle, which only needs the
    # sampled channels of x for an entry of gW.
    N, H, W, Cin, Cout, p, r = 512, 32, 32, 4352, 64, 8, 4
    gen = torch.Generator(device="cuda").manual_seed(99)
    x = torch.randn((N, H, W, Cin), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    gy = (0.01 * torch.randn((N, H, W, Cout), generator=gen, device="cuda")).to(torch.bfloat16)
    w = (0.02 * torch.randn((Cout, Cin), generator=gen, device="cuda")).to(torch.bfloat16)
    idx = oracle.select_bases(p, r, "l1")
    gx, gW = binding.lbp_wht_backward(x, gy, w, p, idx)
    M = N * H * W
    rng = np.random.default_rng(5)
    tokens = np.unique(np.concatenate([[0, M - 1, M // 2 + 17], rng.integers(0, M, 40)])).astype(np.int64)
    gy_h, w_h = to_host(gy), to_host(w)
    want_gx = oracle.lbp_gx_tokens(gy_h, w_h, p, idx, tokens)
    got_gx = to_host(gx.reshape(M, Cin)[torch.from_numpy(tokens).cuda()])
    assert rel_fro(got_gx, want_gx) <= TOL["bf16"]
    cols = np.unique(np.concatenate([[0, Cin - 1], rng.integers(0, Cin, 6)])).astype(np.int64)
    x_cols = to_host(x[..., torch.from_numpy(cols).cuda()].contiguous())          # [N,H,W,len(cols)]
    co = np.repeat(np.arange(0, Cout, 9, dtype=np.int32), len(cols))
    ci_local = np.tile(np.arange(len(cols), dtype=np.int32), len(co) // len(cols))
    want_gw = oracle.lbp_gw_entries(x_cols, gy_h, p, idx, co, ci_local)
    got_gw = to_host(gW[torch.from_numpy(co.astype(np.int64)).cuda(), torch.from_numpy(cols[ci_local]).cuda()])
    assert rel_fro(got_gw, want_gw) <= TOL["bf16"]
