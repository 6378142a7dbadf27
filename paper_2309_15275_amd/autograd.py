"""A linear layer whose backward pass is LBP-WHT (Algorithm 1), for use inside torch.autograd.

Forward: y = x w^T (+ b) is an ordinary dense product and is left to torch (the method does not
touch it); alongside it the layer's own projection kernel computes x^ = WHT(x; I), and ONLY x^ is
kept for the backward pass (Algorithm 1's second statement depends on x and I alone), so the saved
activation is r/patch^2 of x.  Backward: the library's lbp_wht_backward_preprojected produces
g~x and g~w from x^, g_y and w; there is no fallback if the library is missing.  The bias gradient
is the exact column sum of g_y (the paper's layer has no bias, Section 2).

Tensors are token-major: x [N, H, W, Cin], or a token sequence [N, T, Cin] with `grid=(H, W)` whose
last H*W tokens are the grid; T - H*W leading tokens (a class token) are not on the grid and are
treated exactly (their rows of the input gradient and their share of the weight gradient are those
of Eq. 2).  float32 or bfloat16.
"""
import torch

from . import binding


class _LbpWhtLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, patch, basis_idx, profiler=None):
        if x.dim() != 4:
            raise ValueError("x must be [N, H, W, Cin]")
        xc = x.detach().contiguous()
        y = torch.nn.functional.linear(xc, weight, bias)
        ctx.save_for_backward(binding.wht_project(xc, patch, basis_idx), weight)
        ctx.lbp = (int(patch), tuple(int(v) for v in basis_idx), bias is not None)
        ctx.profiler = profiler
        return y

    @staticmethod
    def backward(ctx, gy):
        x_r, weight = ctx.saved_tensors
        patch, basis_idx, has_bias = ctx.lbp
        gy = gy.contiguous()
        if ctx.profiler is not None:
            ctx.profiler(gy, None)
        want_gx, want_gw = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        gx = gW = None
        if want_gx or want_gw:
            gx, gW = binding.lbp_wht_backward_preprojected(
                x_r, gy, weight.detach(), patch, basis_idx, want_gx=want_gx, want_gw=want_gw,
                gw_dtype=weight.dtype)
        gb = gy.sum(dim=(0, 1, 2)) if has_bias and ctx.needs_input_grad[2] else None
        return gx, gW, gb, None, None, None


class _LbpWhtLinearTokensFn(torch.autograd.Function):
    """The same for token sequences [N, T, Cin] with T - H*W tokens in front of the grid."""

    @staticmethod
    def forward(ctx, x, weight, bias, patch, basis_idx, grid, profiler=None):
        if x.dim() != 3:
            raise ValueError("x must be [N, T, Cin]")
        xc = x.detach().contiguous()
        y = torch.nn.functional.linear(xc, weight, bias)
        ctx.save_for_backward(binding.wht_project_tokens(xc, grid, patch, basis_idx), weight)
        ctx.lbp = (int(patch), tuple(int(v) for v in basis_idx), bias is not None, (int(grid[0]), int(grid[1])))
        ctx.profiler = profiler
        return y

    @staticmethod
    def backward(ctx, gy):
        x_r, weight = ctx.saved_tensors
        patch, basis_idx, has_bias, grid = ctx.lbp
        gy = gy.contiguous()
        if ctx.profiler is not None:
            ctx.profiler(gy, grid)
        want_gx, want_gw = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        gx = gW = None
        if want_gx or want_gw:
            gx, gW = binding.lbp_wht_backward_tokens_preprojected(
                x_r, gy, weight.detach(), grid, patch, basis_idx, want_gx=want_gx, want_gw=want_gw,
                gw_dtype=weight.dtype)
        gb = gy.sum(dim=(0, 1)) if has_bias and ctx.needs_input_grad[2] else None
        return gx, gW, gb, None, None, None, None


def lbp_wht_linear(x, weight, bias, patch, basis_idx, grid=None, profiler=None):
    """Functional form: y = x w^T + b with the LBP-WHT backward.  x [N,H,W,Cin], or [N,T,Cin] with grid=(H,W).
    profiler(gy, grid), when given, is called with the output gradient at the start of every backward."""
    if x.dim() == 3:
        if grid is None:
            raise ValueError("a [N, T, C] input needs grid=(H, W)")
        return _LbpWhtLinearTokensFn.apply(x, weight, bias, patch, basis_idx, grid, profiler)
    return _LbpWhtLinearFn.apply(x, weight, bias, patch, basis_idx, profiler)


class LBPWHTLinear(torch.nn.Module):
    """torch.nn.Linear with the LBP-WHT backward.  `order` / `rank` choose a low-pass selection
    (Eq. 8 / Eq. 9); `set_bases` installs any other list; `lhe_profile_steps` > 0 profiles the spectrum
    of g_y for that many backward passes and then switches to the low-heuristic-error selection."""

    def __init__(self, in_features, out_features, bias=True, patch=8, rank=8, order="l1", device=None,
                 dtype=None, lhe_profile_steps=0):
        super().__init__()
        self.in_features, self.out_features, self.patch = in_features, out_features, patch
        # Low-heuristic-error selection (Section 3.2): the WHT spectrum of g_y is accumulated over the
        # first `lhe_profile_steps` backward passes (which run with the low-pass selection), then
        # the `rank` strongest bases replace it.  0: keep the low-pass selection.
        self.rank = rank
        self.lhe_steps_left = int(lhe_profile_steps)
        self.lhe_energy = None
        self.weight = torch.nn.Parameter(torch.empty(out_features, in_features, device=device, dtype=dtype))
        self.bias = torch.nn.Parameter(torch.zeros(out_features, device=device, dtype=dtype)) if bias else None
        torch.nn.init.normal_(self.weight, std=0.02)
        self.basis_idx = tuple(binding.select_bases(patch, rank, order))

    def set_bases(self, basis_idx):
        self.basis_idx = tuple(int(v) for v in basis_idx)

    def _profile(self, gy, grid):
        """Adds one backward pass to the spectrum; switches to the strongest bases when profiling ends."""
        if self.lhe_steps_left <= 0:
            return
        self.lhe_energy = binding.wht_energy(gy, self.patch, energy=self.lhe_energy, grid=grid)
        self.lhe_steps_left -= 1
        if self.lhe_steps_left == 0:
            self.set_bases(binding.select_lhe(self.lhe_energy.cpu().tolist(), self.patch, self.rank))

    def forward(self, x, grid=None):
        if x.dim() == 3:
            if grid is None:
                raise ValueError("a [N, T, C] input needs grid=(H, W)")
            if grid[0] * grid[1] > x.shape[1]:
                raise ValueError("fewer tokens than the grid holds")
            return lbp_wht_linear(x, self.weight, self.bias, self.patch, self.basis_idx, grid, self._profiler())
        return lbp_wht_linear(x, self.weight, self.bias, self.patch, self.basis_idx, None, self._profiler())

    def _profiler(self):
        return self._profile if self.lhe_steps_left > 0 else None
