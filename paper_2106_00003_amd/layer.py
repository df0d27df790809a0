"""PyTorch autograd front end of the library: U(theta) applied to a batch of column vectors as a
differentiable operation (the training use the paper targets: Section 1 and the problem statement of
Section 2 — "forward" builds or applies U, "backward" turns dL/dY into dL/dtheta).

Marshalling only.  forward() is one givens_forward / givens_build call; backward() is one
givens_backward call on the saved *output* (the reverse sweep undoes the rotations, so no
activations other than Y are kept).  For float32 the forward pass prepares the coefficient tables of both
sweep directions once (givens_prepare) and the backward pass reuses them -- theta cannot change in
between; if another call on the stream has replaced the tables meanwhile, the backward pass falls back to
the plain call, which rebuilds them.  There is no CPU path: tensors must live on the GPU.
"""
from __future__ import annotations

import torch

from . import binding


def _plain(n: int, m) -> bool:
    """True when the unrestricted entry points cover the problem (even n, every pair free)."""
    return n % 2 == 0 and (m is None or m == n - 1)


def _prepare(th, n, m, want_backward: bool, B: int) -> int:
    """Token of the prepared tables of th (float32), or 0 when the prepared path does not apply."""
    if th.dtype != torch.float32:
        return 0
    directions = binding.PREPARE_FORWARD
    if want_backward:
        # wide batches take the Gram form, whose dX sweep needs tables of its own
        directions |= binding.PREPARE_BACKWARD_WIDE if B >= 2 * (n + n % 2) else binding.PREPARE_BACKWARD
    return binding.givens_prepare(th, n, m, directions, batch=B)


def _backward(token, th, Y, g, m, need_dx):
    """dX, dtheta from the prepared tables when they are still there, else from the plain call."""
    if token:
        try:
            return binding.givens_backward_prepared(token, Y, g, th.numel(), want_dx=need_dx)
        except binding.GivensError as err:
            if err.code != binding.ERR_STALE:
                raise
    if m is None:
        return binding.givens_backward(th, Y, g, want_dx=need_dx)
    return binding.givens_backward_restricted(th, Y, g, m, want_dx=need_dx)


class _GivensApply(torch.autograd.Function):
    @staticmethod
    def forward(ctx, theta, X, m):
        th, x = theta.detach().contiguous(), X.detach().contiguous()
        n = x.shape[0]
        ctx.m = None if _plain(n, m) else (n - 1 if m is None else m)
        ctx.token = _prepare(th, n, ctx.m, any(ctx.needs_input_grad), x.shape[1])
        if ctx.token:
            Y = binding.givens_forward_prepared(ctx.token, x)
        else:
            Y = binding.givens_forward(th, x) if ctx.m is None else binding.givens_forward_restricted(th, x, ctx.m)
        ctx.save_for_backward(theta, Y)
        return Y

    @staticmethod
    @torch.autograd.function.once_differentiable
    def backward(ctx, G):
        theta, Y = ctx.saved_tensors
        need_dx = ctx.needs_input_grad[1]
        th, g = theta.detach().contiguous(), G.contiguous()
        dX, dtheta = _backward(ctx.token, th, Y, g, ctx.m, need_dx)
        return (dtheta if ctx.needs_input_grad[0] else None), (dX if need_dx else None), None


class _GivensMatrix(torch.autograd.Function):
    @staticmethod
    def forward(ctx, theta, n, m):
        th = theta.detach().contiguous()
        ctx.m = None if _plain(n, m) else (n - 1 if m is None else m)
        ctx.token = _prepare(th, n, ctx.m, ctx.needs_input_grad[0], n)
        if ctx.token:
            U = binding.givens_build_prepared(ctx.token, n, th.device)
        else:
            U = binding.givens_build(th, n) if ctx.m is None else binding.givens_build_restricted(th, n, ctx.m)
        ctx.save_for_backward(theta, U)
        return U

    @staticmethod
    @torch.autograd.function.once_differentiable
    def backward(ctx, G):
        theta, U = ctx.saved_tensors
        th, g = theta.detach().contiguous(), G.contiguous()
        _, dtheta = _backward(ctx.token, th, U, g, ctx.m, False)
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

        self._eval_tables = None  # (token, version of theta, stream) of tables prepared for evaluation

    def forward(self, X: torch.Tensor) -> torch.Tensor:
        if torch.is_grad_enabled() or self.theta.dtype != torch.float32:
            return givens_apply(self.theta, X, self.m)
        # evaluation: the tables of the current theta are prepared once and reused until theta changes
        key = (self.theta._version, self.theta.data_ptr(), torch.cuda.current_stream().cuda_stream)
        x = X.contiguous()
        m = None if _plain(self.n, self.m) else (self.n - 1 if self.m is None else self.m)
        for _ in range(2):
            if self._eval_tables is None or self._eval_tables[1] != key:
                token = binding.givens_prepare(self.theta.detach(), self.n, m, binding.PREPARE_FORWARD)
                self._eval_tables = (token, key)
            try:
                return binding.givens_forward_prepared(self._eval_tables[0], x)
            except binding.GivensError as err:
                if err.code != binding.ERR_STALE:
                    raise
                self._eval_tables = None
        raise RuntimeError("prepared tables were replaced twice in a row")

    def matrix(self) -> torch.Tensor:
        return givens_matrix(self.theta, self.n, self.m)
