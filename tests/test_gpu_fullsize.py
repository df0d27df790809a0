"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(KERNEL_AUTO): n = 4096, B = 4096 (near-identity angles) and n = 2048, B = 65536.

The oracle cannot sweep these sizes in test time, so it is asked for what it can compute one by
one, on the same seeded inputs:
  * sampled columns of Y and dX (columns are independent: the oracle's Algorithm 1 run on the
    sampled columns alone gives exactly those columns),
  * sampled components of dtheta from the rank-2 Jacobian form of Section 4.1 (O(n^2 + nB) each),
and the rest is covered by properties that hold at any size: norm preservation, the adjoint
identity <G, U X> = <U^T G, X>, and a vanishing gradient when the upstream gradient equals Y.
"""
import numpy as np
import pytest

from oracle import c_oracle as C
from oracle import givens_oracle as O
from paper_2106_00003_amd import binding, inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_Y, TOL_G = 1e-5, 1e-4


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    binding.set_kernel(binding.KERNEL_AUTO)
    yield
    binding.release()
    torch.cuda.empty_cache()


def _sample_angles(n, rng, count):
    half = n // 2
    picks = {0, half - 1, (n - 2) * half, (n - 1) * half - 1, (n // 2) * half + half // 2,
             1 * half + 1, (n - 3) * half + 63, (n - 3) * half + 64}
    while len(picks) < count:
        picks.add(int(rng.integers(0, (n - 1) * half)))
    return sorted(picks)


@pytest.mark.parametrize("cfg", [4, 5])
def test_full_size_forward_backward(cfg):
    data = inputs.make_inputs(cfg)
    wl = data["workload"]
    n, B = wl.n, wl.B
    th, X, G = data["theta"], data["X"], data["G"]
    print(f"[fullsize] config {cfg}: n={n} B={B} seed={inputs.BASE_SEED + cfg}", flush=True)
    th_d, x_d, g_d = (torch.from_numpy(a).cuda() for a in (th, X, G))
    want_form = binding.FORM_SCALED if wl.theta_dist == "normal0.1" else binding.FORM_LIFTED
    y_d = binding.givens_forward(th_d, x_d)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    assert binding.last_rotation_form() == want_form
    dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    assert binding.last_rotation_form() == want_form
    torch.cuda.synchronize()

    # ---- properties at full size (fp64 accumulation on the device)
    nx, ny = float(x_d.double().norm()), float(y_d.double().norm())
    assert abs(ny - nx) <= 2e-6 * nx
    lhs = float((g_d.double() * y_d.double()).sum())
    rhs = float((dx_d.double() * x_d.double()).sum())
    scale = float(g_d.double().norm()) * nx
    assert abs(lhs - rhs) <= 1e-6 * scale
    assert abs(float(dx_d.double().norm()) - float(g_d.double().norm())) <= 2e-6 * float(g_d.double().norm())

    # ---- sampled columns against the oracle
    rng = np.random.default_rng(99 + cfg)
    cols = sorted({0, 1, 7, 8, B - 1, B - 9} | {int(c) for c in rng.integers(0, B, 18)})
    pairs = C.schedule(n)
    y_cols = y_d[:, cols].cpu().numpy()
    dx_cols = dx_d[:, cols].cpu().numpy()
    want_y = C.forward(th, X[:, cols], pairs=pairs)
    want_dx = C.grad_operand(th, G[:, cols], pairs=pairs)
    err_y, err_dx = O.rel_fro(y_cols, want_y), O.rel_fro(dx_cols, want_dx)
    print(f"[fullsize] config {cfg}: Y err {err_y:.3e} ({len(cols)} columns), dX err {err_dx:.3e}", flush=True)
    assert err_y <= TOL_Y
    assert err_dx <= TOL_G

    # ---- sampled gradient components against the rank-2 Jacobian form
    x64, g64 = X.astype(np.float64), G.astype(np.float64)
    angles = _sample_angles(n, rng, 14)
    want = np.array([O.grad_theta_single(th, x64, g64, e, pairs=pairs) for e in angles])
    got = dth_d.cpu().numpy()[angles].astype(np.float64)
    err_dth = float(np.linalg.norm(got - want) / np.linalg.norm(want))
    print(f"[fullsize] config {cfg}: dtheta err {err_dth:.3e} on {len(angles)} sampled angles", flush=True)
    assert err_dth <= TOL_G
    del x64, g64

    # ---- upstream gradient equal to the output: gradient of a constant
    _, dth0_d = binding.givens_backward(th_d, y_d, y_d.clone(), want_dx=False)
    typical = float(dth_d.double().abs().mean())
    worst = float(dth0_d.abs().max())
    print(f"[fullsize] config {cfg}: max |dtheta| with G = Y: {worst:.3e} (typical |dtheta| {typical:.3e})",
          flush=True)
    assert worst <= 1e-3 * typical
