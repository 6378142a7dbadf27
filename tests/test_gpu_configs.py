"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (default paths, planner-chosen tiles).  Where the whole oracle takes seconds the
comparison is element by element; at the larger sizes it is on sampled gx rows and gW entries
that the oracle computes one by one, plus properties that hold at any size."""
import os

import numpy as np
import pytest
import torch

import oracle
from _gpu_util import TOL, device_inputs, rel_fro, to_host
from paper_2309_15275_amd import binding, workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    yield
    os.environ.pop("LBP_GEMM_GROUP", None)
    os.environ.pop("LBP_WHT_PATH", None)
    torch.cuda.synchronize()


def sample_indices(wl, seed, n_tokens=48, n_entries=192):
    rng = np.random.default_rng(seed)
    M = wl.tokens
    tokens = np.unique(np.concatenate([[0, M - 1, wl.W - 1, wl.H * wl.W - 1, wl.H * wl.W],
                                       rng.integers(0, M, n_tokens)])).astype(np.int64)
    co = np.concatenate([[0, wl.Cout - 1, 0, wl.Cout - 1], rng.integers(0, wl.Cout, n_entries)]).astype(np.int32)
    ci = np.concatenate([[0, wl.Cin - 1, wl.Cin - 1, 0], rng.integers(0, wl.Cin, n_entries)]).astype(np.int32)
    return tokens, co, ci


def check_sampled(wl, host, gx, gW, idx, seed):
    tokens, co, ci = sample_indices(wl, seed)
    gx_rows = to_host(gx.reshape(-1, wl.Cin)[torch.from_numpy(tokens).cuda()])
    gw_vals = to_host(gW[torch.from_numpy(co.astype(np.int64)).cuda(), torch.from_numpy(ci.astype(np.int64)).cuda()])
    want_gx = oracle.lbp_gx_tokens(host["gy"], host["w"], wl.patch, idx, tokens)
    want_gw = oracle.lbp_gw_entries(host["x"], host["gy"], wl.patch, idx, co, ci)
    return rel_fro(gx_rows, want_gx), rel_fro(gw_vals, want_gw)


def test_cfg2_vitb_fc1_whole_oracle():
    wl = workloads.WORKLOADS["cfg2_vitb_fc1"]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, 8, "l1")
    gx, gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
    gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], wl.patch, idx)
    egx, egw = rel_fro(to_host(gx), gx0), rel_fro(to_host(gW), gW0)
    assert egx <= TOL["bf16"] and egw <= TOL["bf16"], (egx, egw)


def test_cfg2_full_rank_backward_sampled():
    wl = workloads.WORKLOADS["cfg2_vitb_fc1"]
    host, dev = device_inputs(wl)
    gx, gW = binding.full_bp_backward(dev["x"], dev["gy"], dev["w"])
    tokens, co, ci = sample_indices(wl, 21)
    gx_rows = to_host(gx.reshape(-1, wl.Cin)[torch.from_numpy(tokens).cuda()])
    gw_vals = to_host(gW[torch.from_numpy(co.astype(np.int64)).cuda(), torch.from_numpy(ci.astype(np.int64)).cuda()])
    assert rel_fro(gx_rows, oracle.full_gx_tokens(host["gy"], host["w"], tokens)) <= 5e-3
    assert rel_fro(gw_vals, oracle.full_gw_entries(host["x"], host["gy"], co, ci)) <= 5e-3


def test_cfg3_thin_channels_whole_oracle():
    wl = workloads.WORKLOADS["cfg3_effformer_early"]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, 8, "l1")
    gx, gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
    gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], wl.patch, idx)
    egx, egw = rel_fro(to_host(gx), gx0), rel_fro(to_host(gW), gW0)
    assert egx <= TOL["bf16"] and egw <= TOL["bf16"], (egx, egw)


@pytest.mark.parametrize("r", [8, 36])
def test_49_token_maps_whole_oracle(r):
    # 7 x 7 grids inside one zero-padded 8 x 8 patch each, at the channel counts of Section 3.3's example
    wl = workloads.WORKLOADS["pad_7x7_fc2"]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, r, "l1")
    gx, gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
    gx0, gW0 = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], wl.patch, idx)
    egx, egw = rel_fro(to_host(gx), gx0), rel_fro(to_host(gW), gW0)
    assert egx <= TOL["bf16"] and egw <= TOL["bf16"], (egx, egw)


@pytest.mark.parametrize("layer", ["cfg4_vitl_fc1", "cfg4_vitl_fc2"])
def test_cfg4_vitl_rank_sweep(layer):
    wl = workloads.WORKLOADS[layer]
    host, dev = device_inputs(wl)
    for r in wl.ranks:
        idx = oracle.select_bases(wl.patch, r, "l1")
        gx, gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
        if r <= 4:
            gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], wl.patch, idx)
            egx, egw = rel_fro(to_host(gx), gx0), rel_fro(to_host(gW), gW0)
        else:
            egx, egw = check_sampled(wl, host, gx, gW, idx, 40 + r)
        assert egx <= TOL["bf16"] and egw <= TOL["bf16"], (layer, r, egx, egw)


def test_cfg5_attnproj_orders_and_ranks():
    wl = workloads.WORKLOADS["cfg5_vitb_attnproj"]
    host, dev = device_inputs(wl)
    # the two low-pass orders pick the same SET at r = 4, 8, 64 and differ only at r = 16
    for r in (4, 8, 64):
        assert sorted(binding.select_bases(8, r, "l1")) == sorted(binding.select_bases(8, r, "linf"))
    assert sorted(binding.select_bases(8, 16, "l1")) != sorted(binding.select_bases(8, 16, "linf"))
    for r, order in [(4, "l1"), (8, "l1"), (8, "linf"), (16, "l1"), (16, "linf"), (64, "l1")]:
        idx = np.asarray(binding.select_bases(wl.patch, r, order))
        assert np.array_equal(idx, oracle.select_bases(wl.patch, r, order))
        gx, gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
        egx, egw = check_sampled(wl, host, gx, gW, idx, 60 + r)
        assert egx <= TOL["bf16"] and egw <= TOL["bf16"], (r, order, egx, egw)
        if r == 64:
            # all bases kept: the result is exact backpropagation (Eq. 2)
            tokens, co, ci = sample_indices(wl, 99)
            gx_rows = to_host(gx.reshape(-1, wl.Cin)[torch.from_numpy(tokens).cuda()])
            gw_vals = to_host(gW[torch.from_numpy(co.astype(np.int64)).cuda(),
                                 torch.from_numpy(ci.astype(np.int64)).cuda()])
            assert rel_fro(gx_rows, oracle.full_gx_tokens(host["gy"], host["w"], tokens)) <= TOL["bf16"]
            assert rel_fro(gw_vals, oracle.full_gw_entries(host["x"], host["gy"], co, ci)) <= TOL["bf16"]
            gxf, gWf = binding.full_bp_backward(dev["x"], dev["gy"], dev["w"])
            assert rel_fro(to_host(gW), to_host(gWf)) <= TOL["bf16"]
            del gxf, gWf


def test_rank_one_is_pool_matmul_upsample_at_full_size():
    # property that holds at any size: r = 1 (the constant basis) gives gx constant inside every patch
    wl = workloads.WORKLOADS["cfg2_vitb_fc1"]
    host, dev = device_inputs(wl)
    gx, _ = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, [0], want_gw=False)
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
    os.environ["LBP_GEMM_GROUP"] = "0"
    gx0, gW0 = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
    os.environ.pop("LBP_GEMM_GROUP")
    gx1, gW1 = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], wl.patch, idx)
    assert rel_fro(to_host(gx1), to_host(gx0)) <= TOL["bf16"] and rel_fro(to_host(gW1), to_host(gW0)) <= 1e-5
    for gx, gW in ((gx0, gW0), (gx1, gW1)):
        if wl.H % wl.patch or wl.W % wl.patch:
            gxo, gWo = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], wl.patch, idx)
            egx, egw = rel_fro(to_host(gx), gxo), rel_fro(to_host(gW), gWo)
        else:
            egx, egw = check_sampled(wl, host, gx, gW, idx, 77 + case)
        assert egx <= TOL["bf16"] and egw <= TOL["bf16"], (egx, egw)


@pytest.mark.parametrize("path", ["auto", "mfma"])
def test_tensors_beyond_two_to_the_31_elements(path):
    # 2^19 tokens x 4352 channels = 2.28e9 bf16 elements (4.6 GB): element offsets no longer fit 31 bits.
    # The tensor is made on the device (seeded); patches sampled from its whole extent, the last
    # one included, are checked against the oracle's projection of the same values; then the
    # reverse projection of those coefficients, again against the oracle on sampled patches.
    os.environ["LBP_WHT_PATH"] = path
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
    os.environ.pop("LBP_WHT_PATH", None)


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
