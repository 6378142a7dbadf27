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


# Tolerances of the contract: relative Frobenius error against the double-precision oracle.
TOL = {"f32": 1e-5, "bf16": 2e-2}
