"""CPU-only tests of the library's host side: it loads without a GPU, exports every symbol the
header declares, selects bases bit-exactly like the oracle, and reports every argument error
before touching the device (so garbage device pointers are safe to pass here)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2309_15275_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2309_15275_amd import build
        build.build(verbose=False)
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "lbp_wht.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:lbp_|full_bp_)\w+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_selection_is_bit_exact_against_the_oracle(lib):
    for p in (2, 4, 8, 16):
        for order in ("l1", "linf"):
            for r in range(1, p * p + 1):
                assert binding.select_bases(p, r, order) == oracle.select_bases(p, r, order).tolist()


def test_selection_errors(lib):
    buf = (ctypes.c_int32 * 4)()
    assert lib.lbp_wht_select_bases(3, 1, 0, buf) == -3
    assert lib.lbp_wht_select_bases(32, 1, 0, buf) == -3
    assert lib.lbp_wht_select_bases(8, 0, 0, buf) == -4
    assert lib.lbp_wht_select_bases(8, 65, 0, buf) == -4
    assert lib.lbp_wht_select_bases(8, 4, 2, buf) == -9
    assert lib.lbp_wht_select_bases(8, 4, 0, None) == -1


P = ctypes.c_void_p
X, GY, W_, GX, GW = 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x50000000   # never dereferenced


def call_backward(lib, shape=None, patch=8, idx=(0, 1, 8, 9), r=None, x=X, gy=GY, w=W_, gx=GX, gw=GW):
    shape = shape or binding.LbpShape(2, 16, 16, 64, 128, 1, 0)
    arr = (ctypes.c_int32 * max(len(idx), 1))(*idx)
    return lib.lbp_wht_backward(P(x) if x else None, P(gy) if gy else None, P(w) if w else None,
                                ctypes.byref(shape), patch, arr, len(idx) if r is None else r,
                                P(gx) if gx else None, P(gw) if gw else None, None)


def test_backward_argument_errors_are_reported_before_any_device_work(lib):
    S = binding.LbpShape
    assert call_backward(lib, x=0) == -1
    assert call_backward(lib, gx=0, gw=0) == -1
    assert call_backward(lib, shape=S(0, 16, 16, 64, 128, 1, 0)) == -2
    assert call_backward(lib, shape=S(2, -12, 16, 64, 128, 1, 0)) == -2
    assert call_backward(lib, shape=S(1 << 15, 1 << 8, 1 << 8, 8, 8, 1, 0)) == -2  # 2^31 tokens
    assert call_backward(lib, patch=3) == -3
    assert call_backward(lib, patch=32) == -3
    assert call_backward(lib, r=0) == -4
    assert call_backward(lib, idx=tuple(range(65)), r=65) == -4
    assert call_backward(lib, idx=(0, 1, 1, 9)) == -5
    assert call_backward(lib, idx=(0, 1, 64, 9)) == -5
    assert call_backward(lib, idx=(0, -1, 8, 9)) == -5
    assert call_backward(lib, shape=S(2, 16, 16, 64, 128, 7, 0)) == -6
    assert call_backward(lib, shape=S(2, 16, 16, 64, 128, 0, 1)) == -6           # bf16 gW of fp32 tensors
    assert call_backward(lib, gx=X) == -7
    assert call_backward(lib, gw=GY + 64) == -7
    assert call_backward(lib, gx=GW) == -7
    assert call_backward(lib, x=X + 2) == -8
    assert call_backward(lib, shape=S(2, 16, 16, 60, 128, 1, 0)) == -8           # Cin % 8 (bf16)
    assert call_backward(lib, shape=S(2, 16, 16, 64, 126, 0, 0)) == -8           # Cout % 4 (fp32)


def test_full_bp_and_projection_argument_errors(lib):
    S = binding.LbpShape
    sh = S(2, 16, 16, 64, 128, 1, 0)
    assert lib.full_bp_backward(None, P(GY), P(W_), ctypes.byref(sh), P(GX), P(GW), None) == -1
    assert lib.full_bp_backward(P(X), P(GY), P(W_), None, P(GX), P(GW), None) == -1
    assert lib.full_bp_backward(P(X), P(GY), P(W_), ctypes.byref(sh), P(X), P(GW), None) == -7
    idx = (ctypes.c_int32 * 2)(0, 1)
    assert lib.lbp_wht_project(None, 2, 16, 16, 64, 1, 8, idx, 2, P(GX), None) == -1
    assert lib.lbp_wht_project(P(X), 2, 16, 16, 64, 1, 8, idx, 2, P(X), None) == -7
    assert lib.lbp_wht_project(P(X), 2, 16, 16, 64, 1, 5, idx, 2, P(GX), None) == -3
    assert lib.lbp_wht_project(P(X), 2, 16, 0, 64, 1, 8, idx, 2, P(GX), None) == -2
    assert lib.lbp_wht_unproject(P(X), 2, 16, 16, 64, 9, 8, idx, 2, P(GX), None) == -6
    assert lib.lbp_wht_unproject(P(X), 2, 16, 16, 64, 1, 8, idx, 3, P(GX), None) in (-5, -4)


def test_preprojected_backward_argument_errors(lib):
    sh = binding.LbpShape(2, 16, 16, 64, 128, 1, 0)
    idx = (ctypes.c_int32 * 4)(0, 1, 8, 9)
    f = lib.lbp_wht_backward_preprojected
    assert f(None, P(GY), P(W_), ctypes.byref(sh), 8, idx, 4, P(GX), P(GW), None) == -1
    assert f(P(X), P(GY), P(W_), ctypes.byref(sh), 8, idx, 0, P(GX), P(GW), None) == -4
    assert f(P(X), P(GY), P(W_), ctypes.byref(sh), 8, idx, 4, P(X), P(GW), None) == -7
    # x_r is only P*r rows long: a buffer right behind it does not overlap it
    rows_r = 2 * 16 * 16 // 64 * 4
    behind = X + rows_r * 64 * 2
    assert f(P(X), P(GY), P(W_), ctypes.byref(sh), 8, idx, 4, P(behind), P(GW), None) in (0, -11)


def test_lhe_selection_is_bit_exact_against_the_oracle(lib):
    rng = np.random.default_rng(5)
    for p in (2, 4, 8, 16):
        for trial in range(6):
            E = rng.random(p * p)
            if trial % 2:
                E = np.round(E * 4) / 4              # many exact ties
            if trial == 4:
                E[:] = 1.0                           # flat spectrum: LP_L1 order
            for r in (1, 3, p, p * p):
                assert binding.select_lhe(E, p, r) == oracle.select_lhe(E, p, r).tolist()
    assert binding.select_lhe(np.ones(64), 8, 10) == oracle.select_bases(8, 10, "l1").tolist()
    arr = (ctypes.c_double * 64)()
    out = (ctypes.c_int32 * 4)()
    assert lib.lbp_wht_select_lhe(arr, 3, 1, out) == -3
    assert lib.lbp_wht_select_lhe(arr, 8, 65, out) == -4
    assert lib.lbp_wht_select_lhe(None, 8, 4, out) == -1
    assert lib.lbp_wht_energy(None, 2, 16, 16, 64, 1, 8, P(GX), None) == -1
    assert lib.lbp_wht_energy(P(X), 2, 0, 16, 64, 1, 8, P(GX), None) == -2
    assert lib.lbp_wht_energy_workspace_bytes(2, 16, 16, 64, 1, 8) >= 2 * 256 * 64 * 2
    assert lib.lbp_wht_energy_workspace_bytes(2, 16, 16, 64, 1, 5) == 0


def test_no_cpu_fallback_without_a_device(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    assert call_backward(lib) == -11           # valid arguments, no device: HIP error, not a result
    assert lib.lbp_last_hip_error() != 0


def test_workspace_bytes_and_strerror(lib):
    sh = binding.LbpShape(64, 16, 16, 768, 3072, 1, 0)
    need = binding.workspace_bytes(sh, 8, 8)
    Mr = 64 * 256 // 64 * 8
    assert need >= Mr * (3072 + 768) * 2 + Mr * 768 * 4 + 3072 * 768 * 4
    assert binding.workspace_bytes(binding.LbpShape(64, 16, 16, 768, 3072, 5, 0), 8, 8) == 0
    assert binding.workspace_bytes(sh, 8, 0) == 0
    assert binding.workspace_bytes(sh, 0, 0) > 0
    for code in range(0, -12, -1):
        assert binding.strerror(code) and "unknown status" not in binding.strerror(code)
    assert "unknown status" in binding.strerror(-99)


def test_token_sequence_entry_points_check_their_arguments(lib):
    sh = binding.LbpShape(2, 14, 14, 64, 128, 1, 0)
    idx = (ctypes.c_int32 * 4)(0, 1, 8, 9)
    f = lib.lbp_wht_backward_tokens
    args = lambda extra, x=X, gx=GX, r=4: (P(x) if x else None, P(GY), P(W_), ctypes.byref(sh), extra, 8, idx, r,
                                           P(gx) if gx else None, P(GW), None)
    assert f(*args(1, x=0)) == -1
    assert f(*args(-1)) == -2
    assert f(*args(1, r=0)) == -4
    # gx is [N][1 + 196][Cin]: a buffer that starts inside x's 2*197*64 bf16 values overlaps it
    assert f(*args(1, gx=X + 2 * 196 * 64 * 2)) == -7
    assert f(*args(1, gx=X + 2 * 197 * 64 * 2)) in (0, -11)      # right behind x: no overlap
    g = lib.lbp_wht_project_tokens
    assert g(None, 2, 14, 14, 1, 64, 1, 8, idx, 4, P(GX), None) == -1
    assert g(P(X), 2, 14, 14, -3, 64, 1, 8, idx, 4, P(GX), None) == -2
    assert g(P(X), 2, 14, 14, 1, 64, 1, 8, idx, 4, P(X), None) == -7
    h = lib.lbp_wht_backward_tokens_preprojected
    assert h(P(X), P(GY), P(W_), ctypes.byref(sh), 1, 8, idx, 0, P(GX), P(GW), None) == -4
    # workspace: extra tokens add rows to the projected tensors
    assert binding.workspace_bytes(sh, 8, 4, extra=1) > binding.workspace_bytes(sh, 8, 4)
    assert binding.workspace_bytes(sh, 8, 4, extra=-1) == 0


def test_token_pair_entry_points_check_their_arguments(lib):
    sh = binding.LbpShape(2, 14, 14, 64, 128, 1, 0)
    idx = (ctypes.c_int32 * 4)(0, 1, 8, 9)
    P = ctypes.c_void_p
    X, GY, XR, GYR, W_, GX, GW = (0x10000000 + i * 0x1000000 for i in range(7))
    f = lib.lbp_wht_project_pair_tokens
    assert f(None, P(GY), ctypes.byref(sh), 1, 8, idx, 4, P(XR), P(GYR), None) == -1
    assert f(P(X), P(GY), ctypes.byref(sh), -1, 8, idx, 4, P(XR), P(GYR), None) == -2
    assert f(P(X), P(GY), ctypes.byref(sh), 1, 3, idx, 4, P(XR), P(GYR), None) == -3
    assert f(P(X), P(GY), ctypes.byref(sh), 1, 8, idx, 65, P(XR), P(GYR), None) == -4
    assert f(P(X), P(GY), ctypes.byref(sh), 1, 8, idx, 4, P(X + 64), P(GYR), None) == -7
    assert f(P(X), P(GY), ctypes.byref(sh), 1, 8, idx, 4, P(XR + 4), P(GYR), None) == -8
    assert f(P(X), P(GY), ctypes.byref(sh), 1, 8, idx, 4, P(XR), P(GYR), None) in (0, -11)
    g = lib.lbp_wht_products_tokens
    assert g(P(XR), P(GYR), P(W_), ctypes.byref(sh), 1, 8, idx, 4, None, None, None) == -1
    assert g(P(XR), P(GYR), P(W_), ctypes.byref(sh), -3, 8, idx, 4, P(GX), P(GW), None) == -2
    assert g(P(XR), P(GYR), P(W_), ctypes.byref(sh), 1, 8, idx, 4, P(GX), P(XR), None) == -7
    assert g(P(XR), P(GYR), P(W_), ctypes.byref(sh), 1, 8, idx, 4, P(GX), P(GW), None) in (0, -11)


def test_products_entry_point_checks_its_arguments(lib):
    sh = binding.LbpShape(2, 16, 16, 64, 128, 1, 0)
    idx = (ctypes.c_int32 * 4)(0, 1, 8, 9)
    f = lib.lbp_wht_products
    assert f(None, P(GY), P(W_), ctypes.byref(sh), 8, idx, 4, P(GX), P(GW), None) == -1
    assert f(P(X), P(GY), P(W_), ctypes.byref(sh), 8, idx, 65, P(GX), P(GW), None) == -4
    assert f(P(X), P(GY), P(W_), ctypes.byref(sh), 5, idx, 4, P(GX), P(GW), None) == -3
    # gy_r is only P*r = 32 rows of 128 bf16: an output right behind it does not overlap it
    assert f(P(X), P(GY), P(W_), ctypes.byref(sh), 8, idx, 4, P(GY + 32 * 128 * 2), P(GW), None) in (0, -11)
    assert f(P(X), P(GY), P(W_), ctypes.byref(sh), 8, idx, 4, P(GY + 32 * 128 * 2 - 16), P(GW), None) == -7


def test_launch_plans_of_the_benchmark_configurations(lib):
    # host logic only: what a call would launch on a 256-unit device
    binding.reset_options()
    S = binding.LbpShape
    plan = lambda sh, p, r, order="l1", **kw: binding.describe_plan(sh, p, binding.select_bases(p, r, order), num_cus=256, **kw)
    vitb = S(64, 16, 16, 768, 3072, 1, 0)
    t = plan(vitb, 8, 8)
    assert "register kernel (16 of 64" in t and "one grouped launch" in t and "fused (pooled epilogue)" in t
    assert "gW: tile 128x128 (8 wavefronts), split-K 1;" in t
    assert int(t.rsplit("workspace ", 1)[1].split()[0]) <= binding.workspace_bytes(vitb, 8, 8)
    t = plan(vitb, 8, 15)                               # LP_L1 r=15 cannot be pooled
    assert "matrix-core kernel" in t and "fused (matrix-core epilogue)" in t and "one grouped launch" in t
    t = plan(vitb, 8, 36)                               # large rank: big tiles, split-K, separate kernels
    assert "separate launches" in t and "reverse-projection kernel" in t and "reduction kernel" in t
    t = plan(vitb, 8, 16, "linf")                       # the 4 x 4 square of LP_Linf pools like r=8
    assert "register kernel (16 of 64" in t and "fused (pooled epilogue)" in t
    t = plan(vitb, 8, 4)
    assert "register kernel (4 of 64" in t
    t = plan(S(64, 56, 56, 48, 192, 1, 0), 8, 8)        # thin layer: 64 x 64 tiles for both products
    assert t.count("64x64 (4 wavefronts)") == 2 and "one grouped launch" in t
    t = plan(S(2, 8, 8, 64, 64, 0, 0), 4, 4)            # fp32: plain kernels, nothing fused or grouped
    assert "separate launches" in t and "fp32 64x64" in t and "fused" not in t
    t = plan(vitb, 8, 8, want_gx=False)
    assert "separate launches" in t and "gx:" not in t and "gW:" in t
    # launches of four to eight workgroups per compute unit: one grouped launch if the weight-gradient
    # product is split along its reduction and the input-gradient product keeps its own tile
    t = plan(S(128, 32, 32, 768, 768, 1, 0), 8, 16)     # 131072 tokens x 768 channels: 1536 + 252 workgroups
    assert "one grouped launch" in t and "split-K 7" in t and "fused (matrix-core epilogue)" in t
    t = plan(S(128, 7, 7, 3072, 768, 1, 0), 8, 36)      # 49-token maps
    assert "one grouped launch" in t and "split-K 3" in t
    t = plan(S(32, 16, 16, 4096, 1024, 1, 0), 8, 32)    # the weight-gradient product fills the device alone
    assert "separate launches" in t and "split-K 1;" in t
    # few low-rank rows under a long reduction: the fused input-gradient product is cut into slices that join in the launch
    vitl = S(32, 16, 16, 1024, 4096, 1, 0)
    assert "reduction in 4 slices joined in the launch" in plan(vitl, 8, 4)
    assert "reduction in 2 slices joined in the launch" in plan(vitl, 8, 8)
    assert "joined" not in plan(vitl, 8, 16) and "joined" not in plan(S(32, 16, 16, 4096, 1024, 1, 0), 8, 4)
    assert "reduction in 4 slices joined in the launch" in plan(S(8, 16, 16, 768, 3072, 1, 0), 8, 8)      # a small batch
    assert "joined" not in plan(vitb, 8, 8)
    binding.set_option("LBP_GX_JOIN", "3")
    assert "reduction in 3 slices joined in the launch" in plan(vitb, 8, 8)
    assert binding.workspace_bytes(vitb, 8, 8) >= int(plan(vitb, 8, 8).rsplit("workspace ", 1)[1].split()[0])
    binding.set_option("LBP_GX_JOIN", "1")
    assert "joined" not in plan(vitl, 8, 4)
    binding.set_option("LBP_GX_JOIN", None)
    # the switches change the plan at once (the plan cache is keyed on what they decide)
    grouped = plan(vitb, 8, 8)
    binding.set_option("LBP_GEMM_GROUP", "0")
    assert "separate launches" in plan(vitb, 8, 8)
    binding.set_option("LBP_GEMM_GROUP", None)
    assert plan(vitb, 8, 8) == grouped
    binding.set_option("LBP_FUSE_UNPROJECT", "0")
    assert "fused" not in plan(vitb, 8, 8)
    binding.reset_options()
    assert plan(vitb, 8, 8) == grouped


def test_option_switches_check_their_arguments(lib):
    f = lib.lbp_set_option
    assert f(None, b"0") == -1
    assert f(b"LBP_NO_SUCH_SWITCH", b"0") == -12
    assert f(b"LBP_GEMM_TILE", b"8") == -12 and f(b"LBP_GEMM_TILE", b"x") == -12 and f(b"LBP_GEMM_TILE", b"-1") == -12
    assert f(b"LBP_WHT_PATH", b"fast") == -12 and f(b"LBP_GX_COEF", b"f16") == -12
    assert f(b"LBP_FUSE_UNPROJECT", b"2") == -12 and f(b"LBP_GEMM_GROUP", b"yes") == -12
    assert f(b"LBP_GX_JOIN", b"0") == -12 and f(b"LBP_GX_JOIN", b"9") == -12
    for name, values in (("LBP_WHT_PATH", ("generic", "register", "mfma", "auto")), ("LBP_GEMM_PATH", ("simple", "auto")),
                         ("LBP_GEMM_TILE", tuple(str(i) for i in range(8))), ("LBP_FUSE_UNPROJECT", ("0", "1")),
                         ("LBP_GEMM_GROUP", ("0", "1", "2")), ("LBP_GX_COEF", ("f32", "bf16")),
                         ("LBP_GX_JOIN", tuple(str(i) for i in range(1, 9)))):
        for v in values:
            assert f(name.encode(), v.encode()) == 0, (name, v)
        assert f(name.encode(), None) == 0
    assert "option" in binding.strerror(-12)


def test_plan_description_checks_its_arguments(lib):
    sh = binding.LbpShape(2, 16, 16, 64, 128, 1, 0)
    idx = (ctypes.c_int32 * 4)(0, 1, 8, 9)
    buf = ctypes.create_string_buffer(64)
    f = lib.lbp_wht_describe_plan
    assert f(None, 0, 8, idx, 4, 1, 1, 256, buf, 64) == -1
    assert f(ctypes.byref(sh), 0, 8, idx, 4, 1, 1, 256, None, 64) == -1
    assert f(ctypes.byref(sh), 0, 8, idx, 4, 0, 0, 256, buf, 64) == -1
    assert f(ctypes.byref(sh), 0, 7, idx, 4, 1, 1, 256, buf, 64) == -3
    assert f(ctypes.byref(sh), 0, 8, idx, 0, 1, 1, 256, buf, 64) == -4
    assert f(ctypes.byref(sh), -2, 8, idx, 4, 1, 1, 256, buf, 64) == -2
    assert f(ctypes.byref(sh), 0, 8, idx, 4, 1, 1, 256, buf, 64) == 0
    assert len(buf.value) == 63                          # cut to the buffer, NUL-terminated


def test_reported_workspace_covers_every_plan_on_random_shapes(lib):
    # lbp_wht_workspace_bytes is what a caller who brings the workspace allocates: it must cover the
    # plan of any call with that shape, rank and kind of selection, whichever outputs are asked for
    binding.reset_options()
    rng = np.random.default_rng(2024)
    for _ in range(150):
        patch = int(rng.choice([2, 4, 8, 8, 8, 16]))
        bf16 = bool(rng.integers(0, 2))
        mult = 8 if bf16 else 4
        N, H, W = int(rng.integers(1, 40)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        Cin, Cout = mult * int(rng.integers(1, 300)), mult * int(rng.integers(1, 300))
        extra = int(rng.choice([0, 0, 1, 2]))
        r = int(rng.integers(1, patch * patch + 1))
        idx = rng.permutation(patch * patch)[:r] if rng.integers(0, 2) else oracle.select_bases(patch, r, "l1")
        sh = binding.LbpShape(N, H, W, Cin, Cout, 1 if bf16 else 0, 0)
        need = binding.workspace_bytes(sh, patch, r, extra=extra)
        assert need > 0
        for want_gx, want_gw in ((True, True), (True, False), (False, True)):
            for cus in (256, 304, 64):
                t = binding.describe_plan(sh, patch, idx, extra=extra, want_gx=want_gx, want_gw=want_gw, num_cus=cus)
                used = int(t.rsplit("workspace ", 1)[1].split()[0])
                if cus == 256:      # workspace_bytes plans for the current device, else for 256 units
                    assert used <= need, (N, H, W, Cin, Cout, patch, r, extra, t)


def test_the_public_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own (no C++ , no HIP, no torch types)
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "lbp_wht.h"\n'
                   "int main(void) { lbp_shape_t s = {1, 8, 8, 8, 8, LBP_BF16, LBP_F32}; int32_t idx[4];\n"
                   "  return lbp_wht_select_bases(8, 4, LBP_ORDER_L1, idx) + (int)s.N - 1 + (int)(LBP_STATIC_SCRATCH_BYTES == 0); }\n")
    res = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", os.path.join(ROOT, "include"), str(src)],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_reported_workspace_size_covers_every_plan_under_every_switch(lib):
    # lbp_wht_workspace_bytes is what a caller sizes its own workspace with: no plan of the same shape and rank, with
    # whatever outputs wanted and whatever kernel-choice switch set, may need more (host logic only)
    rng = np.random.default_rng(20261)
    checked = 0
    try:
        for _ in range(250):
            patch = int(rng.choice([4, 8, 8, 8, 16]))
            N = int(rng.integers(1, 70))
            H = max(1, int(rng.integers(1, 5)) * patch + int(rng.choice([0, 0, -1])))
            W = int(rng.integers(1, 5)) * patch
            Cin, Cout = int(rng.integers(1, 520)) * 8, int(rng.integers(1, 520)) * 8
            r = int(rng.integers(1, patch * patch + 1))
            idx = binding.select_bases(patch, r, str(rng.choice(["l1", "linf"])))
            extra = int(rng.choice([0, 0, 1, 2]))
            shape = binding.LbpShape(N, H, W, Cin, Cout, 1, int(rng.integers(0, 2)))
            for name, value in ((None, None), ("LBP_GX_JOIN", str(int(rng.integers(1, 9)))),
                                ("LBP_FUSE_UNPROJECT", str(int(rng.integers(0, 2)))), ("LBP_GEMM_GROUP", str(int(rng.integers(0, 3)))),
                                ("LBP_GX_COEF", str(rng.choice(["f32", "bf16"])))):
                binding.reset_options()
                if name:
                    binding.set_option(name, value)
                have = binding.workspace_bytes(shape, patch, r, extra=extra)
                for want_gx, want_gw in ((True, True), (True, False), (False, True)):
                    text = binding.describe_plan(shape, patch, idx, extra=extra, want_gx=want_gx, want_gw=want_gw, num_cus=256)
                    need = int(text.rsplit("workspace ", 1)[1].split()[0])
                    assert need <= have, (N, H, W, Cin, Cout, patch, r, extra, name, value, want_gx, want_gw, need, have)
                    checked += 1
    finally:
        binding.reset_options()
    assert checked == 250 * 5 * 3
