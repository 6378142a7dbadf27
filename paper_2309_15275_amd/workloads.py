"""Seeded synthetic workloads: shapes of ViT linear layers, values with the spectral
structure the paper reports for the output gradient (energy concentrated in the
low-sequency corner, Section 4.5 / Figure 5).

This module only draws random numbers and shapes them.  It holds none of the method's
arithmetic (no Hadamard matrix, no projection, no matmul) so that the CPU oracle and the
GPU library can both be fed from it without sharing any code of their own.

Recipe (numpy PCG64, `default_rng(seed)`; draw order: x source, W, coarse field, noise):
  x   fp32 configs: N(0,1);  bf16 configs: exact-erf GELU of N(0,1)
  W   fp32 configs: N(0, var = 1/Cin);  bf16 configs: N(0, std = 0.02)
  gy  per (image, channel): a coarse S x S Gaussian field, bilinearly upsampled
      (align-corners) to the H x W token grid, plus white noise
      fp32 configs: S = 2, field std 1, noise std 0.1
      bf16 configs: S = 4, field std 1e-2, noise std 1e-3
Everything is generated in fp32; bf16 configs are then rounded once to bf16
(round-to-nearest-even) and returned as fp32 arrays holding exactly those values, plus
helpers to get the raw 16-bit patterns.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    H: int
    W: int
    Cin: int
    Cout: int
    patch: int
    ranks: tuple          # ranks r the configuration is run at
    orders: tuple         # basis orders: "l1", "linf"
    dtype: str            # "f32" or "bf16"
    seed: int
    extra: int = 0        # tokens per image in front of the grid (class token ...)

    @property
    def tokens(self):
        return self.N * (self.H * self.W + self.extra)

    @property
    def patches(self):
        return self.N * (-(-self.H // self.patch)) * (-(-self.W // self.patch))


# The five configurations the benchmark contract names.  cfg4 is a pair of layers.
WORKLOADS = {
    "cfg1_tiny": Workload("cfg1_tiny", 2, 8, 8, 64, 64, 4, (4, 16), ("l1",), "f32", 1001),
    "cfg2_vitb_fc1": Workload("cfg2_vitb_fc1", 64, 16, 16, 768, 3072, 8, (8,), ("l1",), "bf16", 1002),
    "cfg3_effformer_early": Workload("cfg3_effformer_early", 64, 56, 56, 48, 192, 8, (8,), ("l1",),
                                     "bf16", 1003),
    "cfg4_vitl_fc1": Workload("cfg4_vitl_fc1", 32, 16, 16, 1024, 4096, 8, (4, 8, 16, 32), ("l1",),
                              "bf16", 1004),
    "cfg4_vitl_fc2": Workload("cfg4_vitl_fc2", 32, 16, 16, 4096, 1024, 8, (4, 8, 16, 32), ("l1",),
                              "bf16", 1014),
    "cfg5_vitb_attnproj": Workload("cfg5_vitb_attnproj", 128, 32, 32, 768, 768, 8, (4, 8, 16, 64),
                                   ("l1", "linf"), "bf16", 1005),
    # Beyond the five: the 49-token maps of Section 3.3's worked example, (Cx, Cy, L) = (3072, 768, 49);
    # a 7 x 7 grid inside one zero-padded 8 x 8 patch.
    "pad_7x7_fc2": Workload("pad_7x7_fc2", 128, 7, 7, 3072, 768, 8, (8, 36), ("l1",), "bf16", 1006),
    # ViT-B/16 on 224 x 224 images as the layer really sees it: a class token in front of 14 x 14
    # patch tokens (197 per image); the grid is zero-padded to 16 x 16, the class token kept exact.
    "vitb16_197_fc1": Workload("vitb16_197_fc1", 64, 14, 14, 768, 3072, 8, (8,), ("l1",), "bf16", 1007, 1),
    # The small batches of on-device training (the setting the paper's experiments aim at): config 2 with
    # 8 images and with one.  Few low-rank rows under a long reduction over Cout.
    "vitb_fc1_batch8": Workload("vitb_fc1_batch8", 8, 16, 16, 768, 3072, 8, (8,), ("l1",), "bf16", 1008),
    "vitb_fc1_batch1": Workload("vitb_fc1_batch1", 1, 16, 16, 768, 3072, 8, (8,), ("l1",), "bf16", 1009),
}


def scaled(wl, **kw):
    """A smaller (or otherwise altered) copy of a workload, same recipe and seed."""
    return replace(wl, **kw)


def bf16_bits(a):
    """fp32 array -> uint16 array of bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a):
    return bf16_bits_to_f32(bf16_bits(a)).reshape(np.shape(a))


def _lerp_matrix(dst, src):
    """[dst, src] align-corners linear interpolation weights (src_pos = i*(src-1)/(dst-1))."""
    m = np.zeros((dst, src), dtype=np.float32)
    for i in range(dst):
        pos = 0.0 if dst == 1 else i * (src - 1) / (dst - 1)
        i0 = min(int(np.floor(pos)), src - 1)
        i1 = min(i0 + 1, src - 1)
        a = pos - i0
        m[i, i0] += 1.0 - a
        m[i, i1] += a
    return m


def _gelu_erf(a):
    from scipy.special import erf
    return (0.5 * a * (1.0 + erf(a / np.sqrt(2.0)))).astype(np.float32)


def make_token_inputs(wl, extra):
    """Token sequences of a ViT layer: `extra` tokens (class token ...) in front of the H*W grid
    tokens of make_inputs.  Returns dict(x=[N,extra+H*W,Cin], gy=[N,extra+H*W,Cout], w=[Cout,Cin]);
    the extra tokens are drawn like the grid's (activations through GELU, gradients at the scale of
    the smooth field), from a generator of their own."""
    base = make_inputs(wl)
    rng = np.random.default_rng(wl.seed + 7919)
    f32 = wl.dtype == "f32"
    xe = rng.standard_normal((wl.N, extra, wl.Cin), dtype=np.float32)
    ge = rng.standard_normal((wl.N, extra, wl.Cout), dtype=np.float32) * np.float32(1.0 if f32 else 1e-2)
    if not f32:
        xe, ge = round_to_bf16(_gelu_erf(xe)), round_to_bf16(ge)
    x = np.concatenate([xe, base["x"].reshape(wl.N, wl.H * wl.W, wl.Cin)], axis=1)
    gy = np.concatenate([ge, base["gy"].reshape(wl.N, wl.H * wl.W, wl.Cout)], axis=1)
    return {"x": np.ascontiguousarray(x), "gy": np.ascontiguousarray(gy), "w": base["w"]}


def make_inputs(wl):
    """Returns dict(x=[N,H,W,Cin], gy=[N,H,W,Cout], w=[Cout,Cin]) of fp32 arrays; for a
    bf16 workload every value is exactly representable in bf16."""
    rng = np.random.default_rng(wl.seed)
    N, H, W, Cin, Cout = wl.N, wl.H, wl.W, wl.Cin, wl.Cout
    f32 = wl.dtype == "f32"
    x = rng.standard_normal((N, H, W, Cin), dtype=np.float32)
    if not f32:
        x = _gelu_erf(x)
    w_std = np.float32(1.0 / np.sqrt(Cin)) if f32 else np.float32(0.02)
    w = rng.standard_normal((Cout, Cin), dtype=np.float32) * w_std
    S = 2 if f32 else 4
    field_std = np.float32(1.0 if f32 else 1e-2)
    noise_std = np.float32(0.1 if f32 else 1e-3)
    coarse = rng.standard_normal((N, S, S, Cout), dtype=np.float32) * field_std
    ah, aw = _lerp_matrix(H, S), _lerp_matrix(W, S)
    gy = np.einsum("hs,nstc->nhtc", ah, coarse, optimize=True)
    gy = np.einsum("wt,nhtc->nhwc", aw, gy, optimize=True).astype(np.float32)
    gy += rng.standard_normal((N, H, W, Cout), dtype=np.float32) * noise_std
    if not f32:
        x, w, gy = round_to_bf16(x), round_to_bf16(w), round_to_bf16(gy)
    return {"x": np.ascontiguousarray(x), "gy": np.ascontiguousarray(gy), "w": np.ascontiguousarray(w)}
