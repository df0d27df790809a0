"""GPU tests of the autograd front end: gradients that PyTorch's engine gets from the library equal the
oracle's, PyTorch's own finite-difference gradcheck passes on the fp64 entry points, and a few steps of
gradient descent on the angles reduce a loss."""
import numpy as np
import pytest

from oracle import c_oracle as C
from oracle import givens_oracle as O
from paper_2106_00003_amd import binding, inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    binding.set_kernel(binding.KERNEL_AUTO)
    yield
    binding.release()


def _layer():
    from paper_2106_00003_amd import layer
    return layer


@pytest.mark.parametrize("n,B,seed,dist", [(256, 48, 91, "uniform"), (512, 40, 92, "normal0.1")])
def test_autograd_gradients_match_the_oracle(n, B, seed, dist):
    L = _layer()
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    theta = torch.from_numpy(data["theta"]).cuda().requires_grad_(True)
    X = torch.from_numpy(data["X"]).cuda().requires_grad_(True)
    G = torch.from_numpy(data["G"]).cuda()
    Y = L.givens_apply(theta, X)
    (Y * G).sum().backward()                                   # L = sum(G * U X), the benchmark's loss
    want_y = C.forward(data["theta"], data["X"])
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
    assert O.rel_fro(Y.detach().cpu().numpy(), want_y) <= 1e-5
    assert O.rel_fro(theta.grad.cpu().numpy(), want_dth) <= 1e-4
    assert O.rel_fro(X.grad.cpu().numpy(), want_dx) <= 1e-4


def test_matrix_gradient_matches_algorithm_3():
    L = _layer()
    n = 256
    data = inputs.make_custom(n, n, seed=93)
    theta = torch.from_numpy(data["theta"]).cuda().requires_grad_(True)
    G = torch.from_numpy(data["G"]).cuda()
    U = L.givens_matrix(theta, n)
    (U * G).sum().backward()
    want_u = C.forward(data["theta"], None, n=n)
    want = C.grad_theta_alg3(data["theta"], want_u, data["G"])  # Gamma = G when X = I
    assert O.rel_fro(theta.grad.cpu().numpy(), want) <= 1e-4


def test_gradcheck_on_the_fp64_entry_points():
    L = _layer()
    data = inputs.make_inputs(1)                                # n = 8, B = 4, float64
    theta = torch.from_numpy(data["theta"]).cuda().requires_grad_(True)
    X = torch.from_numpy(data["X"]).cuda().requires_grad_(True)
    assert torch.autograd.gradcheck(L.givens_apply, (theta, X), eps=1e-6, atol=1e-7, rtol=1e-6,
                                    nondet_tol=0.0)
    assert torch.autograd.gradcheck(lambda t: L.givens_matrix(t, 8), (theta,), eps=1e-6, atol=1e-7, rtol=1e-6)


def test_restricted_and_odd_layer_gradients():
    L = _layer()
    from oracle import restricted_oracle as R
    n, m, B = 255, 60, 32
    rng = np.random.default_rng(94)
    pairs = R.free_pairs(n, m)
    th = rng.uniform(-np.pi, np.pi, pairs.shape[0]).astype(np.float32)
    x, g = rng.standard_normal((n, B)).astype(np.float32), rng.standard_normal((n, B)).astype(np.float32)
    theta = torch.from_numpy(th).cuda().requires_grad_(True)
    X = torch.from_numpy(x).cuda().requires_grad_(True)
    Y = L.givens_apply(theta, X, m)
    (Y * torch.from_numpy(g).cuda()).sum().backward()
    want_y = C.forward_pairs(th, x, pairs)
    want_dth, want_dx, _ = C.reverse_sweep_pairs(th, want_y, g, pairs)
    assert O.rel_fro(Y.detach().cpu().numpy(), want_y) <= 1e-5
    assert O.rel_fro(theta.grad.cpu().numpy(), want_dth) <= 1e-4
    assert O.rel_fro(X.grad.cpu().numpy(), want_dx) <= 1e-4
    layer = L.OrthogonalLinear(9, m=4, dtype=torch.float64)
    assert layer.theta.numel() == 4 * 9 - 10
    assert torch.autograd.gradcheck(lambda t: L.givens_matrix(t, 9, 4), (layer.theta,), eps=1e-6, atol=1e-7,
                                    rtol=1e-6)


def test_unitary_function_gradcheck_and_oracle():
    L = _layer()
    from oracle import unitary_oracle as V
    n, B = 8, 3
    rng = np.random.default_rng(95)
    count = n * (n - 1) // 2
    theta = torch.from_numpy(rng.uniform(-np.pi, np.pi, count)).cuda().requires_grad_(True)
    phi = torch.from_numpy(rng.uniform(-np.pi, np.pi, count)).cuda().requires_grad_(True)
    X = torch.from_numpy(rng.standard_normal((n, B)) + 1j * rng.standard_normal((n, B))).cuda().requires_grad_(True)
    assert torch.autograd.gradcheck(L.givens_unitary_apply, (theta, phi, X), eps=1e-6, atol=1e-7, rtol=1e-6)
    g = rng.standard_normal((n, B)) + 1j * rng.standard_normal((n, B))
    Y = L.givens_unitary_apply(theta, phi, X)
    loss = (torch.from_numpy(g).cuda().conj() * Y).real.sum()          # L = Re <G, Y>
    loss.backward()
    th, ph, x = theta.detach().cpu().numpy(), phi.detach().cpu().numpy(), X.detach().cpu().numpy()
    want_dth, want_dph, want_dx, _ = V.reverse_sweep(th, ph, V.forward(th, ph, x), g)
    assert V.rel_fro(theta.grad.cpu().numpy(), want_dth) <= 1e-12
    assert V.rel_fro(phi.grad.cpu().numpy(), want_dph) <= 1e-12
    assert V.rel_fro(X.grad.cpu().numpy(), want_dx) <= 1e-12


def test_gradient_descent_on_the_angles_fits_a_rotation():
    L = _layer()
    torch.manual_seed(5)
    n, B = 256, 128
    target = L.OrthogonalLinear(n, init_std=0.05)
    model = L.OrthogonalLinear(n, init_std=0.0)
    X = torch.randn(n, B, device="cuda")
    with torch.no_grad():
        want = target(X)
    opt = torch.optim.SGD(model.parameters(), lr=5e-4)
    losses = []
    for _ in range(40):
        opt.zero_grad()
        loss = ((model(X) - want) ** 2).sum()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.2 * losses[0]
    u = model.matrix().detach().double()
    assert float((u.T @ u - torch.eye(n, device="cuda", dtype=torch.float64)).norm()) <= 1e-4
