"""ctypes binding of liblbpwht.so (include/lbp_wht.h).  Argument marshalling only: every step of
the backward pass runs in the library's HIP kernels.  PyTorch is used for device memory and
streams, nothing else.  There is no fallback: if the library is not built, or a call fails, an
exception is raised.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liblbpwht.so")

LBP_F32, LBP_BF16 = 0, 1
ORDER_L1, ORDER_LINF = 0, 1
_ORDERS = {"l1": ORDER_L1, "linf": ORDER_LINF, ORDER_L1: ORDER_L1, ORDER_LINF: ORDER_LINF}
_DTYPES = {torch.float32: LBP_F32, torch.bfloat16: LBP_BF16}

# every symbol include/lbp_wht.h declares
EXPORTS = ("lbp_wht_select_bases", "lbp_wht_select_lhe", "lbp_wht_energy", "lbp_wht_energy_workspace_bytes", "lbp_wht_backward", "lbp_wht_backward_preprojected", "lbp_wht_backward_profile", "full_bp_backward", "lbp_wht_project",
           "lbp_wht_project_pair", "lbp_wht_unproject", "lbp_wht_workspace_bytes", "lbp_set_workspace",
           "lbp_release_workspace", "lbp_strerror", "lbp_last_hip_error", "lbp_version",
           "lbp_wht_backward_tokens", "lbp_wht_project_tokens", "lbp_wht_backward_tokens_preprojected",
           "lbp_wht_workspace_bytes_tokens", "lbp_wht_products", "lbp_wht_energy_tokens", "lbp_wht_describe_plan", "lbp_wht_backward_static", "lbp_set_option",
           "lbp_wht_project_pair_tokens", "lbp_wht_products_tokens")


class LbpShape(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("Cin", ctypes.c_int32), ("Cout", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("gw_dtype", ctypes.c_int32)]


class LbpError(RuntimeError):
    def __init__(self, code, message, hip_error=0):
        super().__init__(f"liblbpwht: {message} (status {code}, hip error {hip_error})")
        self.code = code
        self.hip_error = hip_error


_lib = None


def load():
    """Loads the built library; raises if it is missing (build with __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -m paper_2309_15275_amd.build` (needs hipcc)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    shp = ctypes.POINTER(LbpShape)
    lib.lbp_wht_select_bases.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p]
    lib.lbp_wht_backward.argtypes = [vp, vp, vp, shp, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp]
    lib.lbp_wht_backward_static.argtypes = lib.lbp_wht_backward.argtypes
    lib.lbp_wht_select_lhe.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int, ctypes.c_int, i32p]
    lib.lbp_wht_energy.argtypes = [vp] + [ctypes.c_int] * 6 + [vp, vp]
    lib.lbp_wht_energy_tokens.argtypes = [vp] + [ctypes.c_int] * 7 + [vp, vp]
    lib.lbp_wht_energy_workspace_bytes.argtypes = [ctypes.c_int] * 6
    lib.lbp_wht_energy_workspace_bytes.restype = ctypes.c_size_t
    lib.lbp_wht_backward_preprojected.argtypes = [vp, vp, vp, shp, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp]
    lib.lbp_wht_describe_plan.argtypes = [shp, ctypes.c_int, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
    lib.lbp_wht_products.argtypes = [vp, vp, vp, shp, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp]
    lib.lbp_wht_backward_profile.argtypes = [vp, vp, vp, shp, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp,
                                             ctypes.POINTER(ctypes.c_float)]
    lib.full_bp_backward.argtypes = [vp, vp, vp, shp, vp, vp, vp]
    lib.lbp_wht_project.argtypes = [vp] + [ctypes.c_int] * 6 + [i32p, ctypes.c_int, vp, vp]
    lib.lbp_wht_unproject.argtypes = [vp] + [ctypes.c_int] * 6 + [i32p, ctypes.c_int, vp, vp]
    lib.lbp_wht_project_pair.argtypes = [vp, vp, shp, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp]
    lib.lbp_wht_project_pair_tokens.argtypes = [vp, vp, shp, ctypes.c_int, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp]
    lib.lbp_wht_products_tokens.argtypes = [vp, vp, vp, shp, ctypes.c_int, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp]
    lib.lbp_wht_backward_tokens.argtypes = [vp, vp, vp, shp, ctypes.c_int, ctypes.c_int, i32p, ctypes.c_int, vp, vp, vp]
    lib.lbp_wht_backward_tokens_preprojected.argtypes = lib.lbp_wht_backward_tokens.argtypes
    lib.lbp_wht_project_tokens.argtypes = [vp] + [ctypes.c_int] * 7 + [i32p, ctypes.c_int, vp, vp]
    lib.lbp_wht_workspace_bytes_tokens.argtypes = [shp, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.lbp_wht_workspace_bytes_tokens.restype = ctypes.c_size_t
    lib.lbp_wht_workspace_bytes.argtypes = [shp, ctypes.c_int, ctypes.c_int]
    lib.lbp_wht_workspace_bytes.restype = ctypes.c_size_t
    lib.lbp_set_workspace.argtypes = [vp, ctypes.c_size_t]
    lib.lbp_release_workspace.argtypes = []
    lib.lbp_set_option.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    lib.lbp_strerror.argtypes = [ctypes.c_int]
    lib.lbp_strerror.restype = ctypes.c_char_p
    lib.lbp_last_hip_error.argtypes = []
    lib.lbp_version.argtypes = []
    for name in EXPORTS:
        getattr(lib, name)          # AttributeError here means the library is stale
    _lib = lib
    return lib


def _check(code):
    if code != 0:
        lib = load()
        raise LbpError(code, lib.lbp_strerror(code).decode(), lib.lbp_last_hip_error())


def strerror(code):
    return load().lbp_strerror(int(code)).decode()


def version():
    return int(load().lbp_version())


OPTIONS = ("LBP_WHT_PATH", "LBP_GEMM_PATH", "LBP_GEMM_TILE", "LBP_FUSE_UNPROJECT", "LBP_GEMM_GROUP", "LBP_GX_COEF", "LBP_GX_JOIN")


def set_option(name, value):
    """A kernel-choice switch of the library (tests and measurement); value None restores the default."""
    _check(load().lbp_set_option(name.encode(), None if value is None else str(value).encode()))


def reset_options():
    for name in OPTIONS:
        set_option(name, None)


def _idx_array(basis_idx):
    vals = [int(v) for v in basis_idx]
    return (ctypes.c_int32 * max(len(vals), 1))(*vals), len(vals)


def patch_count(N, H, W, patch):
    """Patches of N zero-padded H x W grids: N * ceil(H/patch) * ceil(W/patch)."""
    return N * (-(-H // patch)) * (-(-W // patch))


def select_bases(patch, r, order="l1"):
    """Low-pass selection of Section 3.2; returns a list of r indices u*patch + v."""
    if order not in _ORDERS:
        _check(-9)
    out = (ctypes.c_int32 * max(int(r), 1))()
    _check(load().lbp_wht_select_bases(int(patch), int(r), _ORDERS[order], out))
    return list(out[:r])


def select_lhe(energy, patch, r):
    """Low-heuristic-error selection of Section 3.2 from a host sequence of patch^2 energies."""
    vals = [float(v) for v in energy]
    arr = (ctypes.c_double * max(len(vals), 1))(*vals)
    if len(vals) != patch * patch:
        raise ValueError("energy must have patch^2 entries")
    out = (ctypes.c_int32 * max(int(r), 1))()
    _check(load().lbp_wht_select_lhe(arr, int(patch), int(r), out))
    return list(out[:r])


def wht_energy(t, patch, energy=None, stream=None, grid=None):
    """Adds the WHT energy spectrum of t [N,H,W,C] to `energy` (float64 device tensor of patch^2
    entries, made and zeroed when not passed).  Returns it.  With grid=(H, W), t is a token sequence
    [N,T,C] whose last H*W tokens are the grid; the others are skipped."""
    if grid is None:
        N, H, W, C = t.shape
        extra = 0
    else:
        N, T, C = t.shape
        H, W = grid
        extra = T - H * W
        if extra < 0:
            raise ValueError("fewer tokens than the grid holds")
    if energy is None:
        energy = torch.zeros(patch * patch, dtype=torch.float64, device=t.device)
    with torch.cuda.device(t.device):
        _check(load().lbp_wht_energy_tokens(_dev_tensor(t, "t"), N, H, W, extra, C, _DTYPES[t.dtype], int(patch),
                                            _dev_tensor(energy, "energy", torch.float64), _stream_ptr(stream)))
    return energy


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_tensor(t, name, dtype=None):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous CUDA/HIP tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}")
    return ctypes.c_void_p(t.data_ptr())


def make_shape(x, gy, w, gw_dtype=torch.float32):
    N, H, W, Cin = x.shape
    Cout = gy.shape[-1]
    if tuple(gy.shape[:3]) != (N, H, W) or tuple(w.shape) != (Cout, Cin):
        raise ValueError("shapes must be x[N,H,W,Cin], gy[N,H,W,Cout], w[Cout,Cin]")
    if x.dtype not in _DTYPES or gw_dtype not in _DTYPES:
        raise TypeError("dtype must be float32 or bfloat16")
    return LbpShape(N, H, W, Cin, Cout, _DTYPES[x.dtype], _DTYPES[gw_dtype])


def lbp_wht_backward(x, gy, w, patch, basis_idx, gx=None, gW=None, want_gx=True, want_gw=True,
                     gw_dtype=torch.float32, stream=None):
    """Algorithm 1 on the GPU.  x [N,H,W,Cin], gy [N,H,W,Cout], w [Cout,Cin] device tensors of one
    dtype (float32 or bfloat16).  Returns (gx, gW); outputs are allocated when not passed in."""
    shape = make_shape(x, gy, w, gw_dtype)
    if want_gx and gx is None:
        gx = torch.empty_like(x)
    if want_gw and gW is None:
        gW = torch.empty(w.shape, dtype=gw_dtype, device=w.device)
    idx, r = _idx_array(basis_idx)
    with torch.cuda.device(x.device):
        _check(load().lbp_wht_backward(
            _dev_tensor(x, "x"), _dev_tensor(gy, "gy", x.dtype), _dev_tensor(w, "w", x.dtype),
            ctypes.byref(shape), int(patch), idx, r,
            _dev_tensor(gx, "gx", x.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


STATIC_SCRATCH_BYTES = 32 << 20


def lbp_wht_backward_static(x, gy, w, patch, basis_idx, gx, gW, stream=None):
    """lbp_wht_backward through the library's fixed scratch array: the library allocates nothing.
    The caller brings both outputs (either may be None to skip it)."""
    gw_dtype = gW.dtype if gW is not None else torch.float32
    shape = make_shape(x, gy, w, gw_dtype)
    idx, r = _idx_array(basis_idx)
    with torch.cuda.device(x.device):
        _check(load().lbp_wht_backward_static(
            _dev_tensor(x, "x"), _dev_tensor(gy, "gy", x.dtype), _dev_tensor(w, "w", x.dtype),
            ctypes.byref(shape), int(patch), idx, r,
            _dev_tensor(gx, "gx", x.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


def lbp_wht_backward_preprojected(x_r, gy, w, patch, basis_idx, gx=None, gW=None, want_gx=True,
                                  want_gw=True, gw_dtype=torch.float32, stream=None):
    """Algorithm 1 with x^ = WHT(x; I) kept from the forward pass: x_r is [P*r, Cin] (wht_project of
    x with the same basis_idx); gy [N,H,W,Cout], w [Cout,Cin].  Returns (gx, gW)."""
    N, H, W, Cout = gy.shape
    Cin = w.shape[1]
    idx, r = _idx_array(basis_idx)
    if tuple(x_r.shape) != (patch_count(N, H, W, patch) * r, Cin) or tuple(w.shape) != (Cout, Cin):
        raise ValueError("shapes must be x_r[P*r,Cin], gy[N,H,W,Cout], w[Cout,Cin]")
    shape = LbpShape(N, H, W, Cin, Cout, _DTYPES[gy.dtype], _DTYPES[gw_dtype])
    if want_gx and gx is None:
        gx = torch.empty((N, H, W, Cin), dtype=gy.dtype, device=gy.device)
    if want_gw and gW is None:
        gW = torch.empty(w.shape, dtype=gw_dtype, device=w.device)
    with torch.cuda.device(gy.device):
        _check(load().lbp_wht_backward_preprojected(
            _dev_tensor(x_r, "x_r", gy.dtype), _dev_tensor(gy, "gy"), _dev_tensor(w, "w", gy.dtype),
            ctypes.byref(shape), int(patch), idx, r,
            _dev_tensor(gx, "gx", gy.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


def lbp_wht_products(x_r, gy_r, w, grid_shape, patch, basis_idx, gx=None, gW=None, want_gx=True, want_gw=True,
                     gw_dtype=torch.float32, stream=None):
    """Statements 3-6 of Algorithm 1 from projected tensors: x_r [P*r,Cin], gy_r [P*r,Cout] (wht_project_pair),
    w [Cout,Cin]; grid_shape = (N, H, W) of the token grids.  Returns (gx [N,H,W,Cin], gW)."""
    N, H, W = grid_shape
    Cout, Cin = w.shape
    idx, r = _idx_array(basis_idx)
    rows = patch_count(N, H, W, patch) * r
    if tuple(x_r.shape) != (rows, Cin) or tuple(gy_r.shape) != (rows, Cout):
        raise ValueError("shapes must be x_r[P*r,Cin], gy_r[P*r,Cout], w[Cout,Cin]")
    shape = LbpShape(N, H, W, Cin, Cout, _DTYPES[gy_r.dtype], _DTYPES[gw_dtype])
    if want_gx and gx is None:
        gx = torch.empty((N, H, W, Cin), dtype=gy_r.dtype, device=gy_r.device)
    if want_gw and gW is None:
        gW = torch.empty(w.shape, dtype=gw_dtype, device=w.device)
    with torch.cuda.device(gy_r.device):
        _check(load().lbp_wht_products(
            _dev_tensor(x_r, "x_r", gy_r.dtype), _dev_tensor(gy_r, "gy_r"), _dev_tensor(w, "w", gy_r.dtype),
            ctypes.byref(shape), int(patch), idx, r,
            _dev_tensor(gx, "gx", gy_r.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


def _token_shape(t, gy, w, grid, gw_dtype):
    """LbpShape and the number of extra tokens of sequences t/gy [N, T, C] whose last H*W tokens are the grid."""
    N, T = gy.shape[:2]
    H, W = grid
    Cout, Cin = w.shape
    extra = T - H * W
    if gy.dim() != 3 or extra < 0 or gy.shape[2] != Cout:
        raise ValueError("gy must be [N, extra + H*W, Cout] with grid = (H, W)")
    return LbpShape(N, H, W, Cin, Cout, _DTYPES[gy.dtype], _DTYPES[gw_dtype]), extra


def lbp_wht_backward_tokens(x, gy, w, grid, patch, basis_idx, gx=None, gW=None, want_gx=True, want_gw=True,
                            gw_dtype=torch.float32, stream=None):
    """Algorithm 1 on token sequences x [N,T,Cin], gy [N,T,Cout] whose last H*W tokens are the
    grid = (H, W); the T - H*W leading tokens (class token ...) are treated exactly.  Returns (gx, gW)."""
    shape, extra = _token_shape(x, gy, w, grid, gw_dtype)
    if tuple(x.shape) != (shape.N, gy.shape[1], shape.Cin):
        raise ValueError("x must be [N, T, Cin]")
    if want_gx and gx is None:
        gx = torch.empty_like(x)
    if want_gw and gW is None:
        gW = torch.empty(w.shape, dtype=gw_dtype, device=w.device)
    idx, r = _idx_array(basis_idx)
    with torch.cuda.device(x.device):
        _check(load().lbp_wht_backward_tokens(
            _dev_tensor(x, "x"), _dev_tensor(gy, "gy", x.dtype), _dev_tensor(w, "w", x.dtype),
            ctypes.byref(shape), extra, int(patch), idx, r,
            _dev_tensor(gx, "gx", x.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


def wht_project_tokens(t, grid, patch, basis_idx, out=None, stream=None):
    """Forward-pass half for x [N,T,C]: the projected grid [P*r, C] followed by the T - H*W leading
    tokens of every image unchanged -> [P*r + N*extra, C]."""
    N, T, C = t.shape
    H, W = grid
    extra = T - H * W
    if extra < 0:
        raise ValueError("fewer tokens than the grid holds")
    idx, r = _idx_array(basis_idx)
    if out is None:
        out = torch.empty((patch_count(N, H, W, patch) * r + N * extra, C), dtype=t.dtype, device=t.device)
    with torch.cuda.device(t.device):
        _check(load().lbp_wht_project_tokens(_dev_tensor(t, "t"), N, H, W, extra, C, _DTYPES[t.dtype], int(patch),
                                             idx, r, _dev_tensor(out, "out", t.dtype), _stream_ptr(stream)))
    return out


def wht_project_pair_tokens(x, gy, grid, patch, basis_idx, x_r=None, gy_r=None, stream=None):
    """Both projections of token sequences x [N,T,Cin], gy [N,T,Cout] in one launch; the T - H*W leading
    tokens of every image follow the coefficient rows (gy's times patch^2).  Returns (x_r, gy_r)."""
    N, T, Cin = x.shape
    Cout = gy.shape[-1]
    H, W = grid
    extra = T - H * W
    if extra < 0 or tuple(gy.shape[:2]) != (N, T):
        raise ValueError("x and gy must be [N, extra + H*W, C]")
    idx, r = _idx_array(basis_idx)
    rows = patch_count(N, H, W, patch) * r + N * extra
    if x_r is None:
        x_r = torch.empty((rows, Cin), dtype=x.dtype, device=x.device)
    if gy_r is None:
        gy_r = torch.empty((rows, Cout), dtype=x.dtype, device=x.device)
    shape = LbpShape(N, H, W, Cin, Cout, _DTYPES[x.dtype], LBP_F32)
    with torch.cuda.device(x.device):
        _check(load().lbp_wht_project_pair_tokens(_dev_tensor(x, "x"), _dev_tensor(gy, "gy", x.dtype), ctypes.byref(shape),
                                                  extra, int(patch), idx, r, _dev_tensor(x_r, "x_r", x.dtype),
                                                  _dev_tensor(gy_r, "gy_r", x.dtype), _stream_ptr(stream)))
    return x_r, gy_r


def lbp_wht_products_tokens(x_r, gy_r, w, grid_shape, extra, patch, basis_idx, gx=None, gW=None, want_gx=True,
                            want_gw=True, gw_dtype=torch.float32, stream=None):
    """Statements 3-6 of Algorithm 1 from wht_project_pair_tokens' tensors; grid_shape = (N, H, W).
    Returns (gx [N, extra + H*W, Cin], gW)."""
    N, H, W = grid_shape
    Cout, Cin = w.shape
    idx, r = _idx_array(basis_idx)
    rows = patch_count(N, H, W, patch) * r + N * extra
    if tuple(x_r.shape) != (rows, Cin) or tuple(gy_r.shape) != (rows, Cout):
        raise ValueError("shapes must be x_r[P*r + N*extra,Cin], gy_r[P*r + N*extra,Cout], w[Cout,Cin]")
    shape = LbpShape(N, H, W, Cin, Cout, _DTYPES[gy_r.dtype], _DTYPES[gw_dtype])
    if want_gx and gx is None:
        gx = torch.empty((N, extra + H * W, Cin), dtype=gy_r.dtype, device=gy_r.device)
    if want_gw and gW is None:
        gW = torch.empty(w.shape, dtype=gw_dtype, device=w.device)
    with torch.cuda.device(gy_r.device):
        _check(load().lbp_wht_products_tokens(
            _dev_tensor(x_r, "x_r", gy_r.dtype), _dev_tensor(gy_r, "gy_r"), _dev_tensor(w, "w", gy_r.dtype),
            ctypes.byref(shape), int(extra), int(patch), idx, r,
            _dev_tensor(gx, "gx", gy_r.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


def lbp_wht_backward_tokens_preprojected(x_r, gy, w, grid, patch, basis_idx, gx=None, gW=None, want_gx=True,
                                         want_gw=True, gw_dtype=torch.float32, stream=None):
    """lbp_wht_backward_tokens with x_r = wht_project_tokens(x) kept from the forward pass."""
    shape, extra = _token_shape(None, gy, w, grid, gw_dtype)
    idx, r = _idx_array(basis_idx)
    rows = patch_count(shape.N, shape.H, shape.W, patch) * r + shape.N * extra
    if tuple(x_r.shape) != (rows, shape.Cin):
        raise ValueError("x_r must be [P*r + N*extra, Cin]")
    if want_gx and gx is None:
        gx = torch.empty((shape.N, gy.shape[1], shape.Cin), dtype=gy.dtype, device=gy.device)
    if want_gw and gW is None:
        gW = torch.empty(w.shape, dtype=gw_dtype, device=w.device)
    with torch.cuda.device(gy.device):
        _check(load().lbp_wht_backward_tokens_preprojected(
            _dev_tensor(x_r, "x_r", gy.dtype), _dev_tensor(gy, "gy"), _dev_tensor(w, "w", gy.dtype),
            ctypes.byref(shape), extra, int(patch), idx, r,
            _dev_tensor(gx, "gx", gy.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


def lbp_wht_backward_profile(x, gy, w, patch, basis_idx, gx, gW, stream=None):
    """lbp_wht_backward bracketed by HIP events; waits, returns the three stage times in ms:
    (projection, weight-gradient product, input-gradient product + reverse projection)."""
    shape = make_shape(x, gy, w, gW.dtype)
    idx, r = _idx_array(basis_idx)
    ms = (ctypes.c_float * 3)()
    with torch.cuda.device(x.device):
        _check(load().lbp_wht_backward_profile(
            _dev_tensor(x, "x"), _dev_tensor(gy, "gy", x.dtype), _dev_tensor(w, "w", x.dtype),
            ctypes.byref(shape), int(patch), idx, r, _dev_tensor(gx, "gx", x.dtype),
            _dev_tensor(gW, "gW"), _stream_ptr(stream), ms))
    return tuple(ms)


def full_bp_backward(x, gy, w, gx=None, gW=None, want_gx=True, want_gw=True,
                     gw_dtype=torch.float32, stream=None):
    """Exact backward of Eq. 2 on the GPU, same conventions as lbp_wht_backward."""
    shape = make_shape(x, gy, w, gw_dtype)
    if want_gx and gx is None:
        gx = torch.empty_like(x)
    if want_gw and gW is None:
        gW = torch.empty(w.shape, dtype=gw_dtype, device=w.device)
    with torch.cuda.device(x.device):
        _check(load().full_bp_backward(
            _dev_tensor(x, "x"), _dev_tensor(gy, "gy", x.dtype), _dev_tensor(w, "w", x.dtype),
            ctypes.byref(shape),
            _dev_tensor(gx, "gx", x.dtype) if gx is not None else None,
            _dev_tensor(gW, "gW", gw_dtype) if gW is not None else None, _stream_ptr(stream)))
    return gx, gW


def wht_project(t, patch, basis_idx, out=None, stream=None):
    """p(.) of Eq. 6: t [N,H,W,C] -> [P*r, C] of the same dtype, unnormalised."""
    N, H, W, C = t.shape
    idx, r = _idx_array(basis_idx)
    if out is None:
        out = torch.empty((patch_count(N, H, W, patch) * r, C), dtype=t.dtype, device=t.device)
    with torch.cuda.device(t.device):
        _check(load().lbp_wht_project(_dev_tensor(t, "t"), N, H, W, C, _DTYPES[t.dtype], int(patch),
                                      idx, r, _dev_tensor(out, "out", t.dtype), _stream_ptr(stream)))
    return out


def wht_project_pair(x, gy, patch, basis_idx, x_r=None, gy_r=None, stream=None):
    """x^ = WHT(x; I) and g^y = WHT(gy; I) in one launch; returns (x_r, gy_r)."""
    N, H, W, Cin = x.shape
    Cout = gy.shape[-1]
    idx, r = _idx_array(basis_idx)
    rows = patch_count(N, H, W, patch) * r
    if x_r is None:
        x_r = torch.empty((rows, Cin), dtype=x.dtype, device=x.device)
    if gy_r is None:
        gy_r = torch.empty((rows, Cout), dtype=x.dtype, device=x.device)
    shape = LbpShape(N, H, W, Cin, Cout, _DTYPES[x.dtype], LBP_F32)
    with torch.cuda.device(x.device):
        _check(load().lbp_wht_project_pair(_dev_tensor(x, "x"), _dev_tensor(gy, "gy", x.dtype),
                                           ctypes.byref(shape), int(patch), idx, r,
                                           _dev_tensor(x_r, "x_r", x.dtype), _dev_tensor(gy_r, "gy_r", x.dtype),
                                           _stream_ptr(stream)))
    return x_r, gy_r


def wht_unproject(coef, shape, dtype, patch, basis_idx, out=None, stream=None):
    """p^-1(.) of Eq. 7 with the 1/patch^2 factor: coef fp32 [P*r, C] -> [N,H,W,C] of `dtype`."""
    N, H, W, C = shape
    idx, r = _idx_array(basis_idx)
    if out is None:
        out = torch.empty((N, H, W, C), dtype=dtype, device=coef.device)
    with torch.cuda.device(coef.device):
        _check(load().lbp_wht_unproject(_dev_tensor(coef, "coef", torch.float32), N, H, W, C,
                                        _DTYPES[dtype], int(patch), idx, r,
                                        _dev_tensor(out, "out", dtype), _stream_ptr(stream)))
    return out


def describe_plan(shape, patch, basis_idx, extra=0, want_gx=True, want_gw=True, num_cus=0):
    """One line of text: what a backward call with these arguments would launch (no device work)."""
    idx, r = _idx_array(basis_idx)
    buf = ctypes.create_string_buffer(1024)
    _check(load().lbp_wht_describe_plan(ctypes.byref(shape), int(extra), int(patch), idx, r, int(want_gx),
                                        int(want_gw), int(num_cus), buf, len(buf)))
    return buf.value.decode()


def workspace_bytes(shape, patch, r, extra=0):
    return int(load().lbp_wht_workspace_bytes_tokens(ctypes.byref(shape), int(extra), int(patch), int(r)))


def set_workspace(buf):
    """buf: a uint8 device tensor to use as workspace, or None for the internal buffer."""
    if buf is None:
        _check(load().lbp_set_workspace(None, 0))
    else:
        with torch.cuda.device(buf.device):
            _check(load().lbp_set_workspace(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size()))


def release_workspace():
    _check(load().lbp_release_workspace())
