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


class _GivensApply(torch.autograd.Function):
    @staticmethod
    def forward(ctx, theta, X):
        Y = binding.givens_forward(theta.detach().contiguous(), X.detach().contiguous())
        ctx.save_for_backward(theta, Y)
        return Y

    @staticmethod
    @torch.autograd.function.once_differentiable
    def backward(ctx, G):
        theta, Y = ctx.saved_tensors
        need_dx = ctx.needs_input_grad[1]
        dX, dtheta = binding.givens_backward(theta.detach().contiguous(), Y, G.contiguous(), want_dx=need_dx)
        return (dtheta if ctx.needs_input_grad[0] else None), (dX if need_dx else None)


class _GivensMatrix(torch.autograd.Function):
    @staticmethod
    def forward(ctx, theta, n):
        U = binding.givens_build(theta.detach().contiguous(), n)
        ctx.save_for_backward(theta, U)
        return U

    @staticmethod
    @torch.autograd.function.once_differentiable
    def backward(ctx, G):
        theta, U = ctx.saved_tensors
        _, dtheta = binding.givens_backward(theta.detach().contiguous(), U, G.contiguous(), want_dx=False)
        return dtheta, None


def givens_apply(theta: torch.Tensor, X: torch.Tensor) -> torch.Tensor:
    """Y = U(theta) X for X of shape (n, B) (columns are the batch); differentiable in theta and X."""
    return _GivensApply.apply(theta, X)


def givens_matrix(theta: torch.Tensor, n: int) -> torch.Tensor:
    """U(theta) itself, n x n; differentiable in theta."""
    return _GivensMatrix.apply(theta, n)


class OrthogonalLinear(torch.nn.Module):
    """Orthogonal layer y = U(theta) x on column batches (n, B), with n(n-1)/2 angles as its parameters
    in the round-robin order E (Section 3).  Angles start near zero (U near the identity)."""

    def __init__(self, n: int, init_std: float = 0.1, device="cuda", dtype=torch.float32):
        super().__init__()
        if n < 2 or n % 2:
            raise ValueError("n must be even and >= 2")
        self.n = n
        self.theta = torch.nn.Parameter(init_std * torch.randn(n * (n - 1) // 2, device=device, dtype=dtype))

    def forward(self, X: torch.Tensor) -> torch.Tensor:
        return givens_apply(self.theta, X)

    def matrix(self) -> torch.Tensor:
        return givens_matrix(self.theta, self.n)
