"""PyTorch autograd front end of the library: U(theta) applied to a batch of column vectors as a
differentiable operation (the training use the paper targets: Section 1 and the problem statement of
Section 2 — "forward" builds or applies U, "backward" turns dL/dY into dL/dtheta).

Marshalling only.  forward() is one givens_forward / givens_build call; backward() is one
givens_backward call on the saved *output* (the reverse sweep undoes the rotations, so no
activations other than Y are kept).  There is no CPU path: tensors must live on the GPU.
"""
from __future__ import annotations

import torch

from . import binding


def _plain(n: int, m) -> bool:
    """True when the unrestricted entry points cover the problem (even n, every pair free)."""
    return n % 2 == 0 and (m is None or m == n - 1)


class _GivensApply(torch.autograd.Function):
    @staticmethod
    def forward(ctx, theta, X, m):
        th, x = theta.detach().contiguous(), X.detach().contiguous()
        n = x.shape[0]
        ctx.m = None if _plain(n, m) else (n - 1 if m is None else m)
        Y = binding.givens_forward(th, x) if ctx.m is None else binding.givens_forward_restricted(th, x, ctx.m)
        ctx.save_for_backward(theta, Y)
        return Y

    @staticmethod
    @torch.autograd.function.once_differentiable
    def backward(ctx, G):
        theta, Y = ctx.saved_tensors
        need_dx = ctx.needs_input_grad[1]
        th, g = theta.detach().contiguous(), G.contiguous()
        if ctx.m is None:
            dX, dtheta = binding.givens_backward(th, Y, g, want_dx=need_dx)
        else:
            dX, dtheta = binding.givens_backward_restricted(th, Y, g, ctx.m, want_dx=need_dx)
        return (dtheta if ctx.needs_input_grad[0] else None), (dX if need_dx else None), None


class _GivensMatrix(torch.autograd.Function):
    @staticmethod
    def forward(ctx, theta, n, m):
        th = theta.detach().contiguous()
        ctx.m = None if _plain(n, m) else (n - 1 if m is None else m)
        U = binding.givens_build(th, n) if ctx.m is None else binding.givens_build_restricted(th, n, ctx.m)
        ctx.save_for_backward(theta, U)
        return U

    @staticmethod
    @torch.autograd.function.once_differentiable
    def backward(ctx, G):
        theta, U = ctx.saved_tensors
        th, g = theta.detach().contiguous(), G.contiguous()
        if ctx.m is None:
            _, dtheta = binding.givens_backward(th, U, g, want_dx=False)
        else:
            _, dtheta = binding.givens_backward_restricted(th, U, g, ctx.m, want_dx=False)
        return dtheta, None, None


class _UnitaryApply(torch.autograd.Function):
    @staticmethod
    def forward(ctx, theta, phi, X):
        Y = binding.givens_unitary_forward(theta.detach().contiguous(), phi.detach().contiguous(),
                                           X.detach().contiguous())
        ctx.save_for_backward(theta, phi, Y)
        return Y

    @staticmethod
    @torch.autograd.function.once_differentiable
    def backward(ctx, G):
        # PyTorch hands a complex output's gradient over as dL/dRe + i dL/dIm for a real loss L, which is
        # the convention of givens_unitary_backward, and expects the same for the complex input X.
        theta, phi, Y = ctx.saved_tensors
        need_dx = ctx.needs_input_grad[2]
        dX, dtheta, dphi = binding.givens_unitary_backward(theta.detach().contiguous(), phi.detach().contiguous(),
                                                           Y, G.contiguous(), want_dx=need_dx)
        return dtheta, dphi, (dX if need_dx else None)


def givens_unitary_apply(theta: torch.Tensor, phi: torch.Tensor, X: torch.Tensor) -> torch.Tensor:
    """Y = U(theta, phi) X for complex X of shape (n, B) (the paper's appendix on U(n)); differentiable in
    theta, phi and X."""
    return _UnitaryApply.apply(theta, phi, X)


def givens_apply(theta: torch.Tensor, X: torch.Tensor, m: int | None = None) -> torch.Tensor:
    """Y = U(theta) X for X of shape (n, B) (columns are the batch); differentiable in theta and X.
    m restricts the parametrisation to the pairs (i, j) with i < m (Section 5); n may be odd."""
    return _GivensApply.apply(theta, X, m)


def givens_matrix(theta: torch.Tensor, n: int, m: int | None = None) -> torch.Tensor:
    """U(theta) itself, n x n; differentiable in theta."""
    return _GivensMatrix.apply(theta, n, m)


class OrthogonalLinear(torch.nn.Module):
    """Orthogonal layer y = U(theta) x on column batches (n, B), with the free angles as its parameters in
    the round-robin order E (Section 3): n(n-1)/2 of them, or m n - m(m+1)/2 with the parametrisation
    restricted to pairs (i, j), i < m (Section 5).  Angles start near zero (U near the identity)."""

    def __init__(self, n: int, m: int | None = None, init_std: float = 0.1, device="cuda", dtype=torch.float32):
        super().__init__()
        if n < 2:
            raise ValueError("n must be >= 2")
        self.n, self.m = n, m
        count = binding.num_angles(n, m)
        self.theta = torch.nn.Parameter(init_std * torch.randn(count, device=device, dtype=dtype))

    def forward(self, X: torch.Tensor) -> torch.Tensor:
        return givens_apply(self.theta, X, self.m)

    def matrix(self) -> torch.Tensor:
        return givens_matrix(self.theta, self.n, self.m)
