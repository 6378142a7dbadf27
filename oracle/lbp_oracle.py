"""ctypes binding of the plain-C oracle (lbp_oracle.c).  TEST INFRASTRUCTURE ONLY.

Argument marshalling and nothing else: every number comes out of the C file, which
states the method (Algorithm 1, Eq. 2, Eq. 6-9, Table 1) in double precision.
Arrays are numpy, C-contiguous; floating-point inputs are converted to float64
(exact for fp32 and bf16 values).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lbp_oracle.c")
_LIB = os.path.join(_HERE, "liblbp_oracle.so")
_lib = None


def build(force=False):
    """Compile lbp_oracle.c with gcc (OpenMP on).  Returns the path of the library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_I32P = ctypes.POINTER(ctypes.c_int32)
_I64P = ctypes.POINTER(ctypes.c_int64)
_I8P = ctypes.POINTER(ctypes.c_int8)
_F64P = ctypes.POINTER(ctypes.c_double)


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_max_threads.restype = ctypes.c_int
        _lib.oracle_set_threads.restype = None
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a, t):
    return a.ctypes.data_as(t) if a is not None else None


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name} rejected its arguments (code {rc})")


def max_threads():
    return int(_load().oracle_max_threads())


def set_threads(n):
    _load().oracle_set_threads(ctypes.c_int(int(n)))


def sylvester(p):
    out = np.zeros((p, p), dtype=np.int8)
    _check(_load().oracle_sylvester(ctypes.c_int(p), _p(out, _I8P)), "oracle_sylvester")
    return out


def walsh(p):
    out = np.zeros((p, p), dtype=np.int8)
    _check(_load().oracle_walsh(ctypes.c_int(p), _p(out, _I8P)), "oracle_walsh")
    return out


def select_bases(p, r, order):
    """order: 0 or 'l1' = LP_L1, 1 or 'linf' = LP_Linf.  Returns int32[r], idx = u*p + v."""
    order = {"l1": 0, "linf": 1}.get(order, order)
    out = np.zeros(max(int(r), 1), dtype=np.int32)
    _check(_load().oracle_select_bases(ctypes.c_int(p), ctypes.c_int(r), ctypes.c_int(order),
                                       _p(out, _I32P)), "oracle_select_bases")
    return out[:r]


def basis_matrix(p, idx):
    idx = _i32(idx)
    out = np.zeros((p * p, len(idx)), dtype=np.int8)
    _check(_load().oracle_basis_matrix(ctypes.c_int(p), ctypes.c_int(len(idx)), _p(idx, _I32P),
                                       _p(out, _I8P)), "oracle_basis_matrix")
    return out


def project(X, p, idx):
    """X: [N,H,W,C] -> [N*(H/p)*(W/p)*r, C], Eq. 6 per patch, unnormalised."""
    X = _f64(X)
    N, H, W, C = X.shape
    idx = _i32(idx)
    r = len(idx)
    out = np.zeros((N * (H // max(p, 1)) * (W // max(p, 1)) * r, C), dtype=np.float64)
    _check(_load().oracle_project(_p(X, _F64P), N, H, W, C, ctypes.c_int(p), ctypes.c_int(r),
                                  _p(idx, _I32P), _p(out, _F64P)), "oracle_project")
    return out


def unproject(Xr, shape, p, idx):
    """Xr: [P*r, C] -> [N,H,W,C], Eq. 7 per patch with the 1/p^2 scale."""
    N, H, W, C = shape
    Xr = _f64(Xr)
    idx = _i32(idx)
    out = np.zeros((N, H, W, C), dtype=np.float64)
    _check(_load().oracle_unproject(_p(Xr, _F64P), N, H, W, C, ctypes.c_int(p),
                                    ctypes.c_int(len(idx)), _p(idx, _I32P), _p(out, _F64P)),
           "oracle_unproject")
    return out


def lbp_wht_backward(x, gy, w, p, idx, want_gx=True, want_gw=True):
    """Algorithm 1.  x [N,H,W,Cin], gy [N,H,W,Cout], w [Cout,Cin] -> (gx, gW) float64."""
    x, gy, w = _f64(x), _f64(gy), _f64(w)
    N, H, W, Cin = x.shape
    Cout = gy.shape[-1]
    assert gy.shape[:3] == x.shape[:3] and w.shape == (Cout, Cin)
    idx = _i32(idx)
    gx = np.zeros((N, H, W, Cin), dtype=np.float64) if want_gx else None
    gW = np.zeros((Cout, Cin), dtype=np.float64) if want_gw else None
    _check(_load().oracle_lbp_wht_backward(_p(x, _F64P), _p(gy, _F64P), _p(w, _F64P), N, H, W,
                                           Cin, Cout, ctypes.c_int(p), _p(idx, _I32P),
                                           ctypes.c_int(len(idx)), _p(gx, _F64P), _p(gW, _F64P)),
           "oracle_lbp_wht_backward")
    return gx, gW


def full_bp_backward(x, gy, w, want_gx=True, want_gw=True):
    """Eq. 2.  Same layouts as lbp_wht_backward."""
    x, gy, w = _f64(x), _f64(gy), _f64(w)
    N, H, W, Cin = x.shape
    Cout = gy.shape[-1]
    assert gy.shape[:3] == x.shape[:3] and w.shape == (Cout, Cin)
    gx = np.zeros((N, H, W, Cin), dtype=np.float64) if want_gx else None
    gW = np.zeros((Cout, Cin), dtype=np.float64) if want_gw else None
    _check(_load().oracle_full_bp_backward(_p(x, _F64P), _p(gy, _F64P), _p(w, _F64P), N, H, W,
                                           Cin, Cout, _p(gx, _F64P), _p(gW, _F64P)),
           "oracle_full_bp_backward")
    return gx, gW


def lbp_gx_tokens(gy, w, p, idx, tokens):
    """Rows of the approximated gx for the listed flat token indices: [len(tokens), Cin]."""
    gy, w = _f64(gy), _f64(w)
    N, H, W, Cout = gy.shape
    Cin = w.shape[1]
    idx = _i32(idx)
    tokens = np.ascontiguousarray(tokens, dtype=np.int64)
    out = np.zeros((len(tokens), Cin), dtype=np.float64)
    _check(_load().oracle_lbp_gx_tokens(_p(gy, _F64P), _p(w, _F64P), N, H, W, Cin, Cout,
                                        ctypes.c_int(p), _p(idx, _I32P), ctypes.c_int(len(idx)),
                                        _p(tokens, _I64P), ctypes.c_int(len(tokens)),
                                        _p(out, _F64P)), "oracle_lbp_gx_tokens")
    return out


def lbp_gw_entries(x, gy, p, idx, co, ci):
    """Entries gW[co[i], ci[i]] of the approximated weight gradient."""
    x, gy = _f64(x), _f64(gy)
    N, H, W, Cin = x.shape
    Cout = gy.shape[-1]
    idx, co, ci = _i32(idx), _i32(co), _i32(ci)
    out = np.zeros(len(co), dtype=np.float64)
    _check(_load().oracle_lbp_gw_entries(_p(x, _F64P), _p(gy, _F64P), N, H, W, Cin, Cout,
                                         ctypes.c_int(p), _p(idx, _I32P), ctypes.c_int(len(idx)),
                                         _p(co, _I32P), _p(ci, _I32P), ctypes.c_int(len(co)),
                                         _p(out, _F64P)), "oracle_lbp_gw_entries")
    return out


def full_gx_tokens(gy, w, tokens):
    gy, w = _f64(gy), _f64(w)
    Cout, Cin = w.shape
    M = gy.size // Cout
    tokens = np.ascontiguousarray(tokens, dtype=np.int64)
    out = np.zeros((len(tokens), Cin), dtype=np.float64)
    _check(_load().oracle_full_gx_tokens(_p(gy, _F64P), _p(w, _F64P), ctypes.c_long(M), Cin, Cout,
                                         _p(tokens, _I64P), ctypes.c_int(len(tokens)),
                                         _p(out, _F64P)), "oracle_full_gx_tokens")
    return out


def full_gw_entries(x, gy, co, ci):
    x, gy = _f64(x), _f64(gy)
    Cin, Cout = x.shape[-1], gy.shape[-1]
    M = x.size // Cin
    co, ci = _i32(co), _i32(ci)
    out = np.zeros(len(co), dtype=np.float64)
    _check(_load().oracle_full_gw_entries(_p(x, _F64P), _p(gy, _F64P), ctypes.c_long(M), Cin,
                                          Cout, _p(co, _I32P), _p(ci, _I32P),
                                          ctypes.c_int(len(co)), _p(out, _F64P)),
           "oracle_full_gw_entries")
    return out


def wht_energy(X, p):
    """Energy of every basis over all patches and channels: float64[p*p], index u*p + v."""
    X = _f64(X)
    N, H, W, C = X.shape
    out = np.zeros(p * p, dtype=np.float64)
    _check(_load().oracle_wht_energy(_p(X, _F64P), N, H, W, C, ctypes.c_int(p), _p(out, _F64P)),
           "oracle_wht_energy")
    return out


def select_lhe(energy, p, r):
    """Low-heuristic-error selection: the r bases of largest energy, by decreasing energy."""
    energy = _f64(energy)
    out = np.zeros(max(int(r), 1), dtype=np.int32)
    _check(_load().oracle_select_lhe(_p(energy, _F64P), ctypes.c_int(p), ctypes.c_int(r), _p(out, _I32P)),
           "oracle_select_lhe")
    return out[:r]


# --------------------------------------------------------------------------------------------
# Token grids that are not multiples of the patch.  The paper's own maps have 7 x 7 = 49 tokens
# (Section 3.3's worked example, the latency tables of the appendix) and does not say how a
# power-of-two transform meets them; the reading taken here: every image's grid is zero-padded
# at the bottom and the right up to the next multiple of p, Algorithm 1 runs on the padded
# grids unchanged (1/p^2 normalisation included), and the rows of g~x that belong to padding
# are dropped.  Each function below is literally pad -> the function above -> crop.
# --------------------------------------------------------------------------------------------

def pad_grid(X, p):
    """[N,H,W,C] -> [N,ceil(H/p)*p,ceil(W/p)*p,C], new tokens zero."""
    X = _f64(X)
    N, H, W, C = X.shape
    return np.pad(X, ((0, 0), (0, -H % p), (0, -W % p), (0, 0)))


def project_padded(X, p, idx):
    return project(pad_grid(X, p), p, idx)


def unproject_padded(Xr, shape, p, idx):
    N, H, W, C = shape
    full = unproject(Xr, (N, H + (-H % p), W + (-W % p), C), p, idx)
    return np.ascontiguousarray(full[:, :H, :W, :])


def lbp_wht_backward_padded(x, gy, w, p, idx, want_gx=True, want_gw=True):
    H, W = x.shape[1:3]
    gx, gW = lbp_wht_backward(pad_grid(x, p), pad_grid(gy, p), w, p, idx, want_gx, want_gw)
    if gx is not None:
        gx = np.ascontiguousarray(gx[:, :H, :W, :])
    return gx, gW


def wht_energy_padded(X, p):
    return wht_energy(pad_grid(X, p), p)


# --------------------------------------------------------------------------------------------
# Token sequences with tokens that are not on the grid.  A ViT layer sees [class token, H*W
# patch tokens] (a distilled model one more); Algorithm 1 is stated for the H x W map only and
# the paper does not say what happens to the others.  The reading taken here: a token outside
# the grid belongs to no patch, so nothing is projected for it and its part of Eq. 2 is kept
# exactly: its row of g~x is g_y,row w, and its outer product g_y,row^T x_row is added to g~w.
# The grid tokens go through Algorithm 1 (zero-padded if the grid is not a multiple of p).
# --------------------------------------------------------------------------------------------

def lbp_wht_backward_tokens(x, gy, w, grid, p, idx, want_gx=True, want_gw=True):
    """x [N,T,Cin], gy [N,T,Cout] with T = extra + H*W, the extra tokens first; grid = (H, W)."""
    x, gy, w = _f64(x), _f64(gy), _f64(w)
    N, T, Cin = x.shape
    H, W = grid
    extra = T - H * W
    if extra < 0 or gy.shape[:2] != (N, T):
        raise ValueError("token count does not match the grid")
    xg = np.ascontiguousarray(x[:, extra:, :]).reshape(N, H, W, Cin)
    gyg = np.ascontiguousarray(gy[:, extra:, :]).reshape(N, H, W, gy.shape[2])
    gxg, gW = lbp_wht_backward_padded(xg, gyg, w, p, idx, want_gx, want_gw)
    gx = None
    if want_gx:
        gx = np.empty_like(x)
        gx[:, extra:, :] = gxg.reshape(N, H * W, Cin)
        gx[:, :extra, :] = gy[:, :extra, :] @ w                    # Eq. 2 for the tokens outside the grid
    if want_gw:
        ge = gy[:, :extra, :].reshape(N * extra, gy.shape[2])
        xe = x[:, :extra, :].reshape(N * extra, Cin)
        gW = gW + ge.T @ xe                                        # their share of Eq. 2's sum over tokens
    return gx, gW


def flop_model(Cx, Cy, L, r):
    """Table 1: dict of FLOPs for vanilla BP, projection, low-rank matmuls, reverse projection."""
    out = (ctypes.c_double * 4)()
    _check(_load().oracle_flop_model(ctypes.c_long(Cx), ctypes.c_long(Cy), ctypes.c_long(L),
                                     ctypes.c_long(r), out), "oracle_flop_model")
    return {"vanilla_bp": out[0], "projection": out[1], "low_rank_mm": out[2],
            "reverse_projection": out[3]}
