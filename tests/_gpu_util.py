"""Helpers of the GPU parity tests: host arrays -> device tensors and back, error measures."""
import numpy as np
import torch

from paper_2309_15275_amd import workloads


def to_device(a, dtype):
    """fp32 numpy array -> device tensor; for 'bf16' the values must already be bf16-exact."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    bits = workloads.bf16_bits(a).reshape(a.shape)
    assert np.array_equal(workloads.bf16_bits_to_f32(bits).reshape(a.shape), a), "input is not bf16-exact"
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_host(t):
    """device tensor -> float64 numpy (exact)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_fro(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def device_inputs(wl):
    host = workloads.make_inputs(wl)
    dev = {k: to_device(v, wl.dtype) for k, v in host.items()}
    return host, dev


def nan_outputs(x_shape, dtype, w_shape, gw_dtype=torch.float32):
    """gx and gW that start as NaN: a region the library never writes stays NaN and fails the
    finiteness check, whatever an earlier call left in the allocator's recycled block."""
    gx = torch.full(tuple(x_shape), float("nan"), dtype=dtype, device="cuda")
    gW = torch.full(tuple(w_shape), float("nan"), dtype=gw_dtype, device="cuda")
    return gx, gW


def lbp_backward(dev, patch, idx, fn=None, gw_dtype=torch.float32, **kw):
    """binding.lbp_wht_backward (or `fn` with the same calling convention) into NaN-filled outputs;
    asserts that every element was written."""
    from paper_2309_15275_amd import binding
    fn = fn or binding.lbp_wht_backward
    gx, gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape, gw_dtype)
    fn(dev["x"], dev["gy"], dev["w"], patch, idx, gx=gx, gW=gW, gw_dtype=gw_dtype, **kw)
    assert bool(torch.isfinite(gx).all()) and bool(torch.isfinite(gW).all()), "an output region was never written"
    return gx, gW


def full_backward(dev, gw_dtype=torch.float32, **kw):
    """binding.full_bp_backward into NaN-filled outputs; asserts that every element was written."""
    from paper_2309_15275_amd import binding
    gx, gW = nan_outputs(dev["x"].shape, dev["x"].dtype, dev["w"].shape, gw_dtype)
    binding.full_bp_backward(dev["x"], dev["gy"], dev["w"], gx=gx, gW=gW, gw_dtype=gw_dtype, **kw)
    assert bool(torch.isfinite(gx).all()) and bool(torch.isfinite(gW).all()), "an output region was never written"
    return gx, gW


def assert_matches(got, want, tol, what=""):
    """Element-by-element comparison of one output tensor with the oracle's.  Three bounds, so that
    a local error cannot hide in the norm of a large tensor:
      * relative Frobenius error of the whole tensor <= tol (the contract's measure);
      * every row (a token of gx, an output channel of gW): |error row| <= tol * max(|oracle row|,
        rms row norm of the oracle) -- one wrong row fails even among 10^5 good ones;
      * every element: |error| <= 8 * tol * rms of the oracle tensor.
    Returns the relative Frobenius error."""
    g = to_host(got) if isinstance(got, torch.Tensor) else np.asarray(got, dtype=np.float64)
    w = np.asarray(want, dtype=np.float64)
    assert g.shape == w.shape, (what, g.shape, w.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite values"
    d = (g - w).reshape(-1, w.shape[-1])
    w2 = w.reshape(-1, w.shape[-1])
    err = float(np.linalg.norm(d) / max(np.linalg.norm(w2), 1e-300))
    assert err <= tol, (what, "relative Frobenius error", err)
    row_err = np.linalg.norm(d, axis=1)
    row_ref = np.linalg.norm(w2, axis=1)
    floor = float(np.sqrt(np.mean(row_ref ** 2)))
    bad = np.nonzero(row_err > tol * np.maximum(row_ref, floor))[0]
    assert bad.size == 0, (what, "rows beyond the bound", bad[:8].tolist(), float(row_err[bad[0]]), float(row_ref[bad[0]]), floor)
    rms = float(np.sqrt(np.mean(w2 ** 2)))
    worst = float(np.abs(d).max()) if d.size else 0.0
    assert worst <= 8 * tol * rms, (what, "largest element error", worst, rms)
    return err


# Tolerances of the contract: relative Frobenius error against the double-precision oracle.
TOL = {"f32": 1e-5, "bf16": 2e-2}
