"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element on
the same seeded inputs.  Sizes here are small enough for the whole oracle to run in seconds but
span several tiles and ragged tails; the full-size configurations are in test_gpu_configs.py.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from _gpu_util import TOL, assert_matches, device_inputs, full_backward, lbp_backward, nan_outputs, rel_fro, to_device, to_host
from paper_2309_15275_amd import binding, workloads
from paper_2309_15275_amd.workloads import Workload

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    yield
    binding.reset_options()
    torch.cuda.synchronize()


def small(name, N, H, W, Cin, Cout, patch, dtype, seed):
    return Workload(name, N, H, W, Cin, Cout, patch, (), ("l1",), dtype, seed)


SELECTIONS = [
    # (patch, basis list builder)
    (8, lambda: oracle.select_bases(8, 8, "l1")),
    (8, lambda: oracle.select_bases(8, 4, "l1")),
    (8, lambda: oracle.select_bases(8, 16, "linf")),
    (8, lambda: oracle.select_bases(8, 32, "l1")),
    (8, lambda: oracle.select_bases(8, 64, "l1")),
    (8, lambda: np.array([0])),
    (8, lambda: np.array([63, 5, 17, 40, 9])),            # arbitrary, unordered (as LHE could give)
    (8, lambda: np.array([16, 0, 2, 18])),                # pooled along W only / H only mix
    (4, lambda: oracle.select_bases(4, 4, "l1")),
    (4, lambda: oracle.select_bases(4, 16, "l1")),
    (4, lambda: np.array([3, 12, 0])),
    (2, lambda: np.array([0, 3])),
    (2, lambda: oracle.select_bases(2, 4, "linf")),
    (16, lambda: oracle.select_bases(16, 8, "l1")),
    (16, lambda: np.array([255, 0, 17, 100])),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("path", ["auto", "generic", "mfma"])
@pytest.mark.parametrize("sel", range(len(SELECTIONS)))
def test_projection_matches_oracle(dtype, path, sel):
    if path == "mfma" and dtype == "f32":
        pytest.skip("the matrix-core form exists for bf16 tensors only")
    patch, mk = SELECTIONS[sel]
    idx = np.asarray(mk())
    binding.set_option("LBP_WHT_PATH", path)
    # ragged: 3 images, non-square grid, channel count that is not a multiple of 64 lanes
    wl = small("proj", 3, 2 * patch, 3 * patch, 40, 72, patch, dtype, 7 + sel)
    host, dev = device_inputs(wl)
    for name in ("x", "gy"):
        got = to_host(binding.wht_project(dev[name], patch, idx))
        want = oracle.project(host[name], patch, idx)
        err = rel_fro(got, want)
        assert err <= (1e-6 if dtype == "f32" else 4e-3), (name, err)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("path", ["auto", "generic", "mfma"])
@pytest.mark.parametrize("sel", range(len(SELECTIONS)))
def test_reverse_projection_matches_oracle(dtype, path, sel):
    if path == "mfma" and dtype == "f32":
        pytest.skip("the matrix-core form exists for bf16 tensors only")
    patch, mk = SELECTIONS[sel]
    idx = np.asarray(mk())
    binding.set_option("LBP_WHT_PATH", path)
    N, H, W, C = 2, 3 * patch, 2 * patch, 56
    rng = np.random.default_rng(100 + sel)
    coef = rng.standard_normal((N * H * W // (patch * patch) * len(idx), C)).astype(np.float32)
    tdtype = torch.float32 if dtype == "f32" else torch.bfloat16
    got = to_host(binding.wht_unproject(torch.from_numpy(coef).cuda(), (N, H, W, C), tdtype, patch, idx))
    want = oracle.unproject(coef, (N, H, W, C), patch, idx)
    err = rel_fro(got, want)
    # the matrix-core form rounds the coefficients to bf16 before the transform and the result after
    assert err <= (1e-6 if dtype == "f32" else 6e-3 if path == "mfma" else 4e-3), err


def run_backward_case(wl, idx, gw_dtype=torch.float32):
    """The whole call into NaN-filled outputs against the whole oracle: norm, every row, every element."""
    host, dev = device_inputs(wl)
    gx, gW = lbp_backward(dev, wl.patch, idx, gw_dtype=gw_dtype)
    gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], wl.patch, idx)
    return assert_matches(gx, gx0, TOL[wl.dtype], "gx"), assert_matches(gW, gW0, TOL[wl.dtype], "gW")


@pytest.mark.parametrize("r", [4, 16])
def test_cfg1_tiny_fp32(r):
    wl = workloads.WORKLOADS["cfg1_tiny"]
    idx = oracle.select_bases(wl.patch, r, "l1")
    egx, egw = run_backward_case(wl, idx)
    assert egx <= TOL["f32"] and egw <= TOL["f32"], (egx, egw)


def test_cfg1_all_bases_is_exact_backprop_fp32():
    wl = workloads.WORKLOADS["cfg1_tiny"]
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(wl.patch, 16, "l1")
    gx, gW = lbp_backward(dev, wl.patch, idx)
    gx0, gW0 = oracle.full_bp_backward(host["x"], host["gy"], host["w"])
    assert_matches(gx, gx0, TOL["f32"], "gx")
    assert_matches(gW, gW0, TOL["f32"], "gW")


RAGGED = [
    # N, H, W, Cin, Cout, patch, r, order
    (3, 16, 24, 72, 200, 8, 8, "l1"),       # tails in every GEMM dimension
    (2, 16, 16, 136, 264, 8, 4, "l1"),
    (1, 8, 8, 8, 8, 8, 8, "l1"),            # a single patch, minimum channels
    (5, 8, 16, 48, 192, 8, 16, "linf"),
    (2, 16, 8, 320, 64, 8, 32, "l1"),
    (2, 8, 8, 64, 96, 8, 64, "l1"),         # all bases
    (2, 8, 12, 40, 24, 4, 4, "l1"),
    (2, 8, 12, 40, 24, 4, 10, "l1"),
    (3, 4, 6, 16, 32, 2, 3, "l1"),
    (1, 32, 16, 24, 40, 16, 10, "l1"),      # patch 16: generic projection kernels
    (8, 16, 16, 72, 136, 8, 10, "l1"),      # r does not divide the GEMM tile: 3 row tiles of 120
    (2, 16, 16, 72, 136, 8, 3, "l1"),
    (2, 16, 16, 72, 136, 8, 21, "l1"),      # no pooling possible: reverse projection not fused
    (6, 16, 32, 264, 520, 8, 8, "l1"),      # several tiles along every GEMM dimension
]

# (LBP_GEMM_PATH, LBP_FUSE_UNPROJECT): tuned kernels, tuned kernels with the reverse projection as
# a kernel of its own, and the plain cross-check kernels
VARIANTS = [("auto", "1"), ("auto", "0"), ("simple", "1"), ("auto+mfma-wht", "0")]


@pytest.mark.parametrize("variant", range(len(VARIANTS)))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(RAGGED)))
def test_backward_matches_oracle_on_ragged_shapes(dtype, case, variant):
    if dtype == "f32" and variant > 0:
        pytest.skip("the fp32 path has one implementation")
    gemm, fuse = VARIANTS[variant]
    if gemm.endswith("+mfma-wht"):          # both projections in their matrix-core form, nothing fused
        gemm = "auto"
        binding.set_option("LBP_WHT_PATH", "mfma")
    binding.set_option("LBP_GEMM_PATH", gemm)
    binding.set_option("LBP_FUSE_UNPROJECT", fuse)
    N, H, W, Cin, Cout, patch, r, order = RAGGED[case]
    wl = small("ragged", N, H, W, Cin, Cout, patch, dtype, 200 + case)
    idx = oracle.select_bases(patch, r, order)
    egx, egw = run_backward_case(wl, idx)
    assert egx <= TOL[dtype] and egw <= TOL[dtype], (egx, egw)


# The reverse projection as a kernel of its own can be fed fp32 split-K slices or one bf16 tensor of
# coefficients (the product rounds once, as the matrix-core reverse kernel does to fp32 input).
@pytest.mark.parametrize("group", ["1", "0"])
@pytest.mark.parametrize("coef", ["bf16", "f32"])
@pytest.mark.parametrize("case", [(2, 16, 16, 72, 136, 8, 21), (6, 16, 32, 264, 520, 8, 36), (3, 24, 16, 136, 200, 8, 15),
                                  (2, 7, 7, 64, 136, 8, 36), (4, 14, 14, 136, 264, 8, 64), (2, 32, 32, 40, 24, 16, 10)])
def test_unfused_reverse_projection_from_bf16_or_fp32_coefficients(case, coef, group):
    N, H, W, Cin, Cout, patch, r = case
    binding.set_option("LBP_FUSE_UNPROJECT", "0")
    binding.set_option("LBP_GX_COEF", coef)
    binding.set_option("LBP_GEMM_GROUP", group)
    wl = small("coef", N, H, W, Cin, Cout, patch, "bf16", 900 + r)
    idx = oracle.select_bases(patch, r, "l1")
    shape = binding.LbpShape(N, H, W, Cin, Cout, binding.LBP_BF16, binding.LBP_F32)
    text = binding.describe_plan(shape, patch, idx)
    assert ("bf16 coefficients" in text) == (coef == "bf16"), text
    host, dev = device_inputs(wl)
    gx, gW = lbp_backward(dev, patch, idx)
    want_gx, want_gw = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], patch, idx)
    assert_matches(gx, want_gx, TOL["bf16"], "gx")
    assert_matches(gW, want_gw, TOL["bf16"], "gW")


# Grids that are not multiples of the patch: zero-padded at the bottom and right (the 49-token maps
# of Section 3.3).  N, H, W, Cin, Cout, patch, basis list
PADDED = [
    (3, 7, 7, 72, 200, 8, lambda: oracle.select_bases(8, 8, "l1")),
    (2, 7, 7, 64, 136, 8, lambda: oracle.select_bases(8, 36, "l1")),       # the paper's largest rank
    (2, 7, 7, 40, 24, 8, lambda: oracle.select_bases(8, 64, "l1")),        # all bases: exact on real tokens
    (2, 10, 13, 48, 72, 4, lambda: oracle.select_bases(4, 4, "l1")),
    (2, 10, 13, 48, 72, 8, lambda: np.array([63, 5, 17, 40, 9])),
    (1, 3, 5, 16, 8, 2, lambda: np.array([0, 3])),
    (2, 17, 30, 24, 40, 16, lambda: oracle.select_bases(16, 10, "l1")),
    (4, 14, 14, 136, 264, 8, lambda: oracle.select_bases(8, 16, "linf")),  # 2 x 2 patches, 6 rows of padding
    (2, 8, 12, 40, 24, 8, lambda: oracle.select_bases(8, 4, "l1")),        # only W is ragged
]


@pytest.mark.parametrize("path", ["auto", "generic", "mfma"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(PADDED)))
def test_projections_on_zero_padded_grids(dtype, case, path):
    if path == "mfma" and dtype == "f32":
        pytest.skip("the matrix-core form exists for bf16 tensors only")
    N, H, W, Cin, Cout, patch, mk = PADDED[case]
    idx = np.asarray(mk())
    binding.set_option("LBP_WHT_PATH", path)
    wl = small("padded", N, H, W, Cin, Cout, patch, dtype, 300 + case)
    host, dev = device_inputs(wl)
    for name in ("x", "gy"):
        got = to_host(binding.wht_project(dev[name], patch, idx))
        want = oracle.project_padded(host[name], patch, idx)
        assert got.shape == want.shape
        assert rel_fro(got, want) <= (1e-6 if dtype == "f32" else 4e-3), name
    xr, gyr = binding.wht_project_pair(dev["x"], dev["gy"], patch, idx)
    assert rel_fro(to_host(xr), oracle.project_padded(host["x"], patch, idx)) <= (1e-6 if dtype == "f32" else 4e-3)
    assert rel_fro(to_host(gyr), oracle.project_padded(host["gy"], patch, idx)) <= (1e-6 if dtype == "f32" else 4e-3)
    rng = np.random.default_rng(400 + case)
    coef = rng.standard_normal((wl.patches * len(idx), Cin)).astype(np.float32)
    tdtype = torch.float32 if dtype == "f32" else torch.bfloat16
    # the output starts as NaN: every real token must be written
    out = torch.full((N, H, W, Cin), float("nan"), dtype=tdtype, device="cuda")
    binding.wht_unproject(torch.from_numpy(coef).cuda(), (N, H, W, Cin), tdtype, patch, idx, out=out)
    want = oracle.unproject_padded(coef, (N, H, W, Cin), patch, idx)
    assert rel_fro(to_host(out), want) <= (1e-6 if dtype == "f32" else 6e-3)
    assert not bool(torch.isnan(out.float()).any())


@pytest.mark.parametrize("variant", [("auto", "1"), ("auto", "0"), ("simple", "1")])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(PADDED)))
def test_backward_on_zero_padded_grids(dtype, case, variant):
    gemm, fuse = variant
    if dtype == "f32" and variant != ("auto", "1"):
        pytest.skip("the fp32 path has one implementation")
    binding.set_option("LBP_GEMM_PATH", gemm)
    binding.set_option("LBP_FUSE_UNPROJECT", fuse)
    N, H, W, Cin, Cout, patch, mk = PADDED[case]
    idx = np.asarray(mk())
    wl = small("padded", N, H, W, Cin, Cout, patch, dtype, 500 + case)
    host, dev = device_inputs(wl)
    # guard rows behind gx: nothing may be written past the last real token
    gx_buf = torch.full((N * H * W + 64, Cin), 7.0, dtype=dev["x"].dtype, device="cuda")
    gx = gx_buf[:N * H * W].view(N, H, W, Cin)
    gx.fill_(float("nan"))                  # every real token must be written
    gW = torch.full((Cout, Cin), float("nan"), dtype=torch.float32, device="cuda")
    binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], patch, idx, gx=gx, gW=gW)
    gx0, gW0 = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], patch, idx)
    assert_matches(gx, gx0, TOL[dtype], "gx")
    assert_matches(gW, gW0, TOL[dtype], "gW")
    assert bool((gx_buf[N * H * W:] == 7.0).all())
    if len(idx) == patch * patch:
        fx, fW = oracle.full_bp_backward(host["x"], host["gy"], host["w"])
        assert_matches(gx, fx, TOL[dtype], "gx against exact backprop")
        assert_matches(gW, fW, TOL[dtype], "gW against exact backprop")
    # x projected ahead of time gives the same bits
    x_r = binding.wht_project(dev["x"], patch, idx)
    gx2, gW2 = nan_outputs(gx.shape, gx.dtype, gW.shape)
    binding.lbp_wht_backward_preprojected(x_r, dev["gy"], dev["w"], patch, idx, gx=gx2, gW=gW2)
    assert torch.equal(gx2, gx) and torch.equal(gW2, gW)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_energy_spectrum_on_a_zero_padded_grid(dtype):
    wl = small("padded-energy", 3, 7, 7, 48, 72, 8, dtype, 77)
    host, dev = device_inputs(wl)
    got = binding.wht_energy(dev["gy"], 8).cpu().numpy()
    want = oracle.wht_energy_padded(host["gy"], 8)
    tol = 1e-5 if dtype == "f32" else 5e-3          # bf16: coefficients are rounded before squaring
    assert np.max(np.abs(got - want)) <= tol * want.max()


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5, 6, 7])
@pytest.mark.parametrize("case", [0, 3, 10, 13])
def test_every_gemm_tile_shape_matches_oracle(case, tile):
    # LBP_GEMM_TILE forces one tile shape of the matrix-core kernel for every product of the call
    binding.set_option("LBP_GEMM_TILE", str(tile))
    N, H, W, Cin, Cout, patch, r, order = RAGGED[case]
    wl = small("tiles", N, H, W, Cin, Cout, patch, "bf16", 400 + case)
    idx = oracle.select_bases(patch, r, order)
    run_backward_case(wl, idx)
    host, dev = device_inputs(wl)
    gx, gW = full_backward(dev)
    gx0, gW0 = oracle.full_bp_backward(host["x"], host["gy"], host["w"])
    assert_matches(gx, gx0, 5e-3, "exact gx")
    assert_matches(gW, gW0, 5e-3, "exact gW")


# (N, H, W, Cin, Cout, patch, r, order, tokens in front of the grid): reductions over Cout long enough to cut
JOINED = [
    (2, 16, 16, 72, 520, 8, 8, "l1", 0),        # pooled epilogue, tails in every dimension
    (3, 16, 24, 136, 776, 8, 4, "l1", 0),
    (2, 16, 16, 72, 520, 8, 21, "l1", 0),       # matrix-core epilogue, 126-row tiles
    (2, 14, 14, 264, 1032, 8, 8, "l1", 1),      # zero-padded grid with a class token
    (4, 7, 7, 136, 512, 8, 15, "l1", 0),        # one padded patch per image
    (6, 16, 32, 264, 1544, 8, 16, "linf", 0),   # several tiles along every dimension
]


@pytest.mark.parametrize("tile", [None, "4"])        # the planner's 64-row tile for the input gradient, or 128 rows for both
@pytest.mark.parametrize("slices", ["2", "3", "8"])
@pytest.mark.parametrize("case", range(len(JOINED)))
def test_input_gradient_reduction_cut_into_slices_that_join_inside_the_launch(case, slices, tile):
    # the fused input-gradient product of a grouped launch with its reduction over Cout in 2, 3 or 8 slices: every
    # slice leaves a partial tile, the last one to finish adds them in slice order and runs the reverse projection
    N, H, W, Cin, Cout, patch, r, order, extra = JOINED[case]
    wl = small("join", N, H, W, Cin, Cout, patch, "bf16", 610 + case)
    idx = oracle.select_bases(patch, r, order)
    if extra:
        host = workloads.make_token_inputs(wl, extra)
        dev = {k: to_device(v, "bf16") for k, v in host.items()}
        want_gx, want_gw = oracle.lbp_wht_backward_tokens(host["x"], host["gy"], host["w"], (H, W), patch, idx)

        def call():
            gx = torch.full((N, extra + H * W, Cin), float("nan"), dtype=dev["x"].dtype, device="cuda")
            gW = torch.full((Cout, Cin), float("nan"), dtype=torch.float32, device="cuda")
            binding.lbp_wht_backward_tokens(dev["x"], dev["gy"], dev["w"], (H, W), patch, idx, gx=gx, gW=gW)
            return gx, gW
    else:
        host, dev = device_inputs(wl)
        want_gx, want_gw = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], patch, idx)

        def call():
            return lbp_backward(dev, patch, idx)
    binding.set_option("LBP_GEMM_TILE", tile)
    binding.set_option("LBP_FUSE_UNPROJECT", "1")
    shape = binding.LbpShape(N, H, W, Cin, Cout, binding.LBP_BF16, binding.LBP_F32)
    # a workspace of the test's own, filled with a byte pattern: what a call writes there can be counted
    binding.set_option("LBP_GX_JOIN", slices)
    space = torch.empty(binding.workspace_bytes(shape, patch, r, extra=extra) + 256, dtype=torch.uint8, device="cuda")
    binding.set_workspace(space)
    try:
        binding.set_option("LBP_GX_JOIN", "1")
        space.fill_(0xCD)
        gx1, gW1 = call()
        torch.cuda.synchronize()
        written_whole = int((space != 0xCD).sum())
        binding.set_option("LBP_GX_JOIN", slices)
        text = binding.describe_plan(shape, patch, idx, extra=extra)
        k_slice = -(-(-(-Cout // int(slices))) // 64) * 64
        cut = k_slice >= 256 and (int(slices) - 1) * k_slice < Cout          # no short and no empty slice
        assert (f"reduction in {slices} slices joined in the launch" in text) == cut, text
        assert "one grouped launch" in text, text
        space.fill_(0xCD)
        gx2, gW2 = call()
        torch.cuda.synchronize()
        written_cut = int((space != 0xCD).sum())
        gx3, gW3 = call()
        torch.cuda.synchronize()
    finally:
        binding.set_workspace(None)
    assert torch.equal(gx2.view(torch.int16), gx3.view(torch.int16))      # whoever finishes a tile last, the same bits
    assert torch.equal(gW1.view(torch.int32), gW2.view(torch.int32))      # the other product is untouched
    # the slices leave their partial tiles in the workspace: a cut reduction writes more of it (else the launch
    # silently ran the reduction in one piece)
    if cut:
        assert written_cut > written_whole + 64 * 128 * 2, (written_whole, written_cut)
    else:
        assert written_cut == written_whole and torch.equal(gx1.view(torch.int16), gx2.view(torch.int16))
    assert_matches(gx2, want_gx, TOL["bf16"], "gx")
    assert_matches(gW2, want_gw, TOL["bf16"], "gW")
    assert_matches(gx1, want_gx, TOL["bf16"], "gx, one slice")


@pytest.mark.parametrize("case,slices", [(1, "2"), (1, "3"), (2, "2"), (5, "2"), (5, "5")])
def test_input_gradient_alone_with_its_reduction_cut_inside_the_launch(case, slices):
    # only g~x wanted: the fused product is a launch of its own and cuts its reduction the same way
    N, H, W, Cin, Cout, patch, r, order, extra = JOINED[case]
    wl = small("join1", N, H, W, Cin, Cout, patch, "bf16", 650 + case)
    idx = oracle.select_bases(patch, r, order)
    host, dev = device_inputs(wl)
    want_gx, _ = oracle.lbp_wht_backward_padded(host["x"], host["gy"], host["w"], patch, idx, want_gw=False)
    shape = binding.LbpShape(N, H, W, Cin, Cout, binding.LBP_BF16, binding.LBP_F32)
    binding.set_option("LBP_FUSE_UNPROJECT", "1")
    binding.set_option("LBP_GX_JOIN", slices)
    text = binding.describe_plan(shape, patch, idx, want_gw=False)
    assert f"reduction in {slices} slices joined in the launch" in text and "gW:" not in text, text
    space = torch.empty(binding.workspace_bytes(shape, patch, r) + 256, dtype=torch.uint8, device="cuda")
    binding.set_workspace(space)
    try:
        written = []
        for join in ("1", slices, slices):
            binding.set_option("LBP_GX_JOIN", join)
            space.fill_(0xCD)
            gx = torch.full_like(dev["x"], float("nan"))
            binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], patch, idx, gx=gx, want_gw=False)
            torch.cuda.synchronize()
            written.append((int((space != 0xCD).sum()), gx))
    finally:
        binding.set_workspace(None)
    assert written[1][0] > written[0][0] + 64 * 128 * 2, [w[0] for w in written]       # the slices' partial tiles
    assert torch.equal(written[1][1].view(torch.int16), written[2][1].view(torch.int16))
    for _, gx in written:
        assert_matches(gx, want_gx, TOL["bf16"], "gx")


@pytest.mark.parametrize("tile", ["4", "6"])
@pytest.mark.parametrize("fuse", ["1", "0"])
@pytest.mark.parametrize("case", [0, 3, 5, 10, 13])
def test_grouped_launch_on_ragged_shapes(case, fuse, tile):
    # tiles 4 and 6 for both products are pairs the grouped kernel covers: one launch runs both; the
    # result must equal the separate launches bit for bit and the oracle within tolerance
    N, H, W, Cin, Cout, patch, r, order = RAGGED[case]
    wl = small("group", N, H, W, Cin, Cout, patch, "bf16", 430 + case)
    idx = oracle.select_bases(patch, r, order)
    host, dev = device_inputs(wl)
    binding.set_option("LBP_GEMM_TILE", tile)
    binding.set_option("LBP_FUSE_UNPROJECT", fuse)
    binding.set_option("LBP_GEMM_GROUP", "0")
    gx0, gW0 = lbp_backward(dev, patch, idx)
    binding.set_option("LBP_GEMM_GROUP", "1")
    gx1, gW1 = lbp_backward(dev, patch, idx)
    assert torch.equal(gx0.view(torch.int16), gx1.view(torch.int16))
    assert torch.equal(gW0.view(torch.int32), gW1.view(torch.int32))
    binding.set_option("LBP_GEMM_GROUP", "2")       # the same launch with the weight-gradient workgroups first
    gx2, gW2 = lbp_backward(dev, patch, idx)
    assert torch.equal(gx0.view(torch.int16), gx2.view(torch.int16))
    assert torch.equal(gW0.view(torch.int32), gW2.view(torch.int32))
    gxo, gWo = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], patch, idx)
    assert_matches(gx1, gxo, TOL["bf16"], "gx")
    assert_matches(gW1, gWo, TOL["bf16"], "gW")


@pytest.mark.parametrize("fuse", ["1", "0"])
@pytest.mark.parametrize("r", [8, 21, 36, 64])
def test_a_non_finite_gradient_stays_inside_its_patch(r, fuse):
    # g~x of a patch depends on g_y of that patch only (Eq. 6, Eq. 7 are per patch): an infinite g_y in one
    # patch may make that patch's g~x non-finite, every other token must keep its bits.  (The fused
    # matrix-core epilogue reads 16 coefficient rows at a time, which at r = 21 or 36 reach into the
    # next patch's rows.)
    binding.set_option("LBP_FUSE_UNPROJECT", fuse)
    wl = small("inf", 3, 16, 24, 136, 264, 8, "bf16", 470 + r)
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(8, r, "l1")
    gx_a, _ = lbp_backward(dev, 8, idx)
    bad = dev["gy"].clone()
    bad[1, 8 + 3, 16 + 5, 7] = float("inf")          # image 1, patch row 1, patch column 2
    gx_b = torch.full_like(dev["x"], float("nan"))
    binding.lbp_wht_backward(dev["x"], bad, dev["w"], 8, idx, gx=gx_b, want_gw=False)
    inside = torch.zeros((3, 16, 24), dtype=torch.bool, device="cuda")
    inside[1, 8:16, 16:24] = True
    assert not bool(torch.isfinite(gx_b[inside]).all())
    assert torch.equal(gx_b[~inside].view(torch.int16), gx_a[~inside].view(torch.int16))


def test_split_k_partial_sums_feed_the_reverse_projection():
    # few rows, long reduction: the planner splits the input-gradient product over K and the
    # reverse-projection kernel adds the slices up
    wl = small("splitgx", 1, 8, 16, 64, 4096, 8, "bf16", 450)
    for r in (4, 21):
        idx = oracle.select_bases(8, r, "l1")
        run_backward_case(wl, idx)


def test_arbitrary_unordered_selection_backward():
    wl = small("lhe", 3, 16, 16, 72, 136, 8, "bf16", 260)
    for idx in ([9, 0, 18, 2, 16], [63, 1, 8], [0, 4, 32, 36]):
        run_backward_case(wl, np.asarray(idx))


@pytest.mark.parametrize("gemm", ["auto", "simple"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_full_rank_backward_matches_oracle(dtype, gemm):
    binding.set_option("LBP_GEMM_PATH", gemm)
    wl = small("full", 3, 16, 24, 72, 200, 8, dtype, 300)
    host, dev = device_inputs(wl)
    gx, gW = full_backward(dev)
    gx0, gW0 = oracle.full_bp_backward(host["x"], host["gy"], host["w"])
    assert_matches(gx, gx0, TOL["f32"] if dtype == "f32" else 5e-3, "gx")
    assert_matches(gW, gW0, TOL["f32"] if dtype == "f32" else 5e-3, "gW")


def test_only_one_output_requested():
    wl = small("one", 2, 16, 16, 64, 128, 8, "bf16", 310)
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(8, 8, "l1")
    gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], 8, idx)
    gx, gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape)
    _, none = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx, gx=gx, want_gw=False)
    assert none is None
    assert_matches(gx, gx0, TOL["bf16"], "gx alone")
    none, _ = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx, gW=gW, want_gx=False)
    assert none is None
    assert_matches(gW, gW0, TOL["bf16"], "gW alone")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_with_x_projected_in_the_forward_pass(dtype):
    # x^ depends only on x and the index set (Alg. 1, first statement): computed once ahead of
    # time it must give the very same bits, and match the oracle's whole Algorithm 1
    wl = small("pre", 3, 16, 24, 72, 200, 8, dtype, 360)
    host, dev = device_inputs(wl)
    for r, order in [(8, "l1"), (21, "l1")]:
        idx = oracle.select_bases(8, r, order)
        x_r = binding.wht_project(dev["x"], 8, idx)
        gx, gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape)
        binding.lbp_wht_backward_preprojected(x_r, dev["gy"], dev["w"], 8, idx, gx=gx, gW=gW)
        gx1, gW1 = lbp_backward(dev, 8, idx)
        assert torch.equal(gx, gx1) and torch.equal(gW, gW1)
        gx0, gW0 = oracle.lbp_wht_backward(host["x"], host["gy"], host["w"], 8, idx)
        assert_matches(gx, gx0, TOL[dtype], "gx")
        assert_matches(gW, gW0, TOL[dtype], "gW")
    # only gW needs x^ at all
    _, gW2 = binding.lbp_wht_backward_preprojected(x_r, dev["gy"], dev["w"], 8, idx, want_gx=False)
    assert torch.equal(gW2, gW)


def test_stage_timing_entry_point_runs_the_same_backward():
    # lbp_wht_backward_profile: the call bracketed by events, products launched one after the other
    wl = small("profile", 4, 16, 16, 136, 264, 8, "bf16", 279)
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(8, 8, "l1")
    binding.set_option("LBP_GEMM_GROUP", "0")
    gx0, gW0 = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
    binding.set_option("LBP_GEMM_GROUP", None)
    gx = torch.full_like(gx0, float("nan"))
    gW = torch.full_like(gW0, float("nan"))
    ms = binding.lbp_wht_backward_profile(dev["x"], dev["gy"], dev["w"], 8, idx, gx, gW)
    assert len(ms) == 3 and all(0.0 < t < 100.0 for t in ms)
    assert torch.equal(gx.view(torch.int16), gx0.view(torch.int16)) and torch.equal(gW.view(torch.int32), gW0.view(torch.int32))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_products_from_projected_tensors_give_the_same_bits(dtype):
    # lbp_wht_products is statements 3-6 of Algorithm 1 on tensors projected by lbp_wht_project_pair
    wl = small("products", 3, 16, 24, 72, 136, 8, dtype, 275)
    host, dev = device_inputs(wl)
    for idx in (oracle.select_bases(8, 8, "l1"), oracle.select_bases(8, 21, "l1")):
        x_r, gy_r = binding.wht_project_pair(dev["x"], dev["gy"], 8, idx)
        a = lbp_backward(dev, 8, idx)
        b = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape)
        binding.lbp_wht_products(x_r, gy_r, dev["w"], (wl.N, wl.H, wl.W), 8, idx, gx=b[0], gW=b[1])
        bits = torch.int32 if dtype == "f32" else torch.int16
        assert torch.equal(a[0].view(bits), b[0].view(bits)) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("patch", [4, 8, 16])
def test_energy_spectrum_matches_oracle(dtype, patch):
    wl = small("energy", 3, 2 * patch, 3 * patch, 40, 72, patch, dtype, 500 + patch)
    host, dev = device_inputs(wl)
    E = binding.wht_energy(dev["gy"], patch)
    E0 = oracle.wht_energy(host["gy"], patch)
    tol = 1e-5 if dtype == "f32" else 5e-3          # bf16: coefficients are rounded before squaring
    assert np.max(np.abs(E.cpu().numpy() - E0)) <= tol * E0.max()
    assert np.allclose(E.cpu().numpy(), E0, rtol=10 * tol, atol=tol * E0.max())
    # a second call accumulates, and repeats the same bits
    E2 = binding.wht_energy(dev["gy"], patch)
    assert torch.equal(E2, E)
    binding.wht_energy(dev["gy"], patch, energy=E)
    assert torch.equal(E, 2 * E2)


def test_lhe_selection_end_to_end():
    # profile gy, pick the r strongest bases, run the backward with them (Section 3.2)
    wl = small("lhe2e", 4, 16, 16, 64, 96, 8, "bf16", 520)
    host, dev = device_inputs(wl)
    E = binding.wht_energy(dev["gy"], 8).cpu().numpy()
    E0 = oracle.wht_energy(host["gy"], 8)
    idx = binding.select_lhe(E, 8, 10)
    idx0 = oracle.select_lhe(E0, 8, 10)
    # the selection is unique only up to near-ties: the energy the chosen set keeps must match
    assert E0[idx].sum() >= (1 - 1e-3) * E0[idx0].sum()
    assert len(set(idx)) == 10 and idx[0] == 0
    run_backward_case(wl, np.asarray(idx))


def test_bf16_weight_gradient_output():
    wl = small("gwbf16", 2, 16, 16, 64, 128, 8, "bf16", 320)
    idx = oracle.select_bases(8, 8, "l1")
    run_backward_case(wl, idx, gw_dtype=torch.bfloat16)


def test_outputs_are_overwritten_and_repeatable():
    wl = small("rep", 2, 16, 16, 64, 128, 8, "bf16", 330)
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(8, 8, "l1")
    gx = torch.full_like(dev["x"], 7.0)
    gW = torch.full((128, 64), -3.0, device="cuda")
    binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx, gx=gx, gW=gW)
    gx2, gW2 = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
    assert torch.equal(gx, gx2) and torch.equal(gW, gW2)      # bit-identical run to run


def test_non_default_stream():
    wl = small("stream", 2, 16, 16, 64, 128, 8, "bf16", 340)
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(8, 8, "l1")
    ref_gx, ref_gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        gx, gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
    s.synchronize()
    assert torch.equal(gx, ref_gx) and torch.equal(gW, ref_gW)


def test_caller_workspace():
    wl = small("ws", 2, 16, 16, 64, 128, 8, "bf16", 350)
    host, dev = device_inputs(wl)
    idx = oracle.select_bases(8, 8, "l1")
    ref_gx, ref_gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
    shape = binding.make_shape(dev["x"], dev["gy"], dev["w"])
    need = binding.workspace_bytes(shape, 8, 8)
    assert need > 0
    buf = torch.empty(need, dtype=torch.uint8, device="cuda")
    try:
        binding.set_workspace(buf)
        gx, gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
        assert torch.equal(gx, ref_gx) and torch.equal(gW, ref_gW)
        binding.set_workspace(buf[:256])
        with pytest.raises(binding.LbpError) as e:
            binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
        assert e.value.code == -10
    finally:
        binding.set_workspace(None)


def test_selection_on_the_library_side_is_bit_exact():
    for p in (2, 4, 8, 16):
        for order in ("l1", "linf"):
            for r in (1, 2, 3, p, p * p // 2, p * p):
                assert binding.select_bases(p, r, order) == oracle.select_bases(p, r, order).tolist()


def test_backward_inside_a_captured_graph_replays_correctly():
    # After one eager call (workspace grown, kernels configured) the call makes no allocation and no
    # synchronisation, so it can be recorded into a HIP graph.  Replays, with new inputs written in place
    # and eager work in between, must reproduce the eager results bit for bit.
    wl = small("graph", 4, 16, 16, 136, 264, 8, "bf16", 77)
    idx = oracle.select_bases(8, 8, "l1")
    host, dev = device_inputs(wl)
    gx = torch.empty_like(dev["x"])
    gW = torch.empty(dev["w"].shape, dtype=torch.float32, device="cuda")
    binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx, gx=gx, gW=gW)      # warm-up, eager
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx, gx=gx, gW=gW)
    for rep in range(4):
        with torch.no_grad():
            dev["gy"].mul_(-0.5 if rep % 2 else 2.0)           # exact in bf16: new inputs, same buffers
            dev["x"].copy_(dev["x"].roll(1, dims=0))
        gx.fill_(float("nan"))
        gW.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got_gx, got_gW = gx.clone(), gW.clone()
        ref_gx, ref_gW = binding.lbp_wht_backward(dev["x"], dev["gy"], dev["w"], 8, idx)
        torch.cuda.synchronize()
        assert torch.equal(got_gx, ref_gx) and torch.equal(got_gW, ref_gW), rep
