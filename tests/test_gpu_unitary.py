"""GPU parity of the unitary extension (the paper's appendix) through the C ABI against oracle/unitary_oracle.py."""
import numpy as np
import pytest

from oracle import givens_oracle as O
from oracle import unitary_oracle as V
from paper_2106_00003_amd import binding

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    yield
    binding.release()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def make(n, B, seed, real, cplx):
    rng = np.random.default_rng(seed)
    count = n * (n - 1) // 2
    theta = rng.uniform(-np.pi, np.pi, count).astype(real)
    phi = rng.uniform(-np.pi, np.pi, count).astype(real)
    x = (rng.standard_normal((n, B)) + 1j * rng.standard_normal((n, B))).astype(cplx)
    g = (rng.standard_normal((n, B)) + 1j * rng.standard_normal((n, B))).astype(cplx)
    return theta, phi, x, g


def check(n, B, seed, real=np.float32, cplx=np.complex64, tol_y=1e-5, tol_g=1e-4, family=None):
    theta, phi, x, g = make(n, B, seed, real, cplx)
    print(f"[unitary] n={n} B={B} seed={seed} dtype={np.dtype(cplx).name} family={family}", flush=True)
    th_d, ph_d = dev(theta), dev(phi)
    y_d = binding.givens_unitary_forward(th_d, ph_d, dev(x))
    assert family is None or binding.last_kernel() == family
    want_y = V.forward_blocks(theta, phi, x)
    err_y = V.rel_fro(host(y_d), want_y)
    dx_d, dth_d, dph_d = binding.givens_unitary_backward(th_d, ph_d, y_d, dev(g))
    assert family is None or binding.last_kernel() == family
    want_dth, want_dph, want_dx, _ = V.reverse_sweep_blocks(theta, phi, want_y, g)
    errs = (err_y, V.rel_fro(host(dx_d), want_dx), V.rel_fro(host(dth_d), want_dth), V.rel_fro(host(dph_d), want_dph))
    print("[unitary]   errors Y %.2e dX %.2e dtheta %.2e dphi %.2e" % errs, flush=True)
    assert errs[0] <= tol_y and max(errs[1:]) <= tol_g
    u_d = binding.givens_unitary_build(th_d, ph_d, n)
    assert family is None or binding.last_kernel() == family
    # the oracle builds all n columns of U up to n = 1024 and a sample of them beyond (columns do not interact)
    cols = np.arange(n) if n <= 1024 else np.unique(np.concatenate([[0, 1, n // 2, n - 1],
                                                                   np.random.default_rng(seed).integers(0, n, 12)]))
    want_u = V.forward_blocks(theta, phi, np.eye(n)[:, cols])
    err_u = V.rel_fro(host(u_d)[:, cols], want_u)
    print("[unitary]   U %.2e on %d columns" % (err_u, cols.size), flush=True)
    assert err_u <= tol_y
    return theta, phi, x, g, host(y_d)


def test_float64_against_the_definition_and_finite_differences():
    n, B = 8, 4
    theta, phi, x, g, y = check(n, B, 401, np.float64, np.complex128, 1e-12, 1e-12)
    u = V.dense_product(n, theta, phi)                                   # explicit factors
    assert V.rel_fro(y, u @ x) <= 1e-12
    _, dth_d, dph_d = binding.givens_unitary_backward(dev(theta), dev(phi), dev(y), dev(g))
    fd_th, fd_ph = V.finite_differences(theta, phi, x, g)
    assert V.rel_fro(host(dth_d), fd_th) <= 1e-7 and V.rel_fro(host(dph_d), fd_ph) <= 1e-7


@pytest.mark.parametrize("n,B,seed", [(2, 1, 411), (4, 3, 412), (34, 19, 413), (130, 40, 414), (256, 64, 415)])
def test_float32_shapes(n, B, seed):
    check(n, B, seed)


def test_n1024_and_in_place():
    n, B = 1024, 20
    theta, phi, x, g, y = check(n, B, 421)
    buf = dev(x)
    binding.givens_unitary_forward(dev(theta), dev(phi), buf, Y=buf)
    assert np.array_equal(host(buf), y)
    g_buf = dev(g)
    dx_d, _, _ = binding.givens_unitary_backward(dev(theta), dev(phi), dev(y), g_buf, dX=g_buf)
    want_dx = V.grad_operand(theta, phi, g) if n <= 64 else None
    u_d = binding.givens_unitary_build(dev(theta), dev(phi), n)
    u = host(u_d).astype(np.complex128)
    assert V.rel_fro(u.conj().T @ u, np.eye(n)) <= 1e-5
    assert V.rel_fro(host(g_buf), u.conj().T @ g.astype(np.complex128)) <= 1e-4


def test_zero_phases_reproduce_the_real_entry_points():
    n, B = 256, 32
    rng = np.random.default_rng(431)
    theta = rng.uniform(-np.pi, np.pi, n * (n - 1) // 2).astype(np.float32)
    x = rng.standard_normal((n, B)).astype(np.float32)
    args = (dev(theta), dev(np.zeros_like(theta)), dev(x.astype(np.complex64)))
    y_car = host(binding.givens_unitary_forward(*args))           # carousel family: phases carried as angles
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    binding.set_kernel(binding.KERNEL_LDS)
    try:
        y_c = host(binding.givens_unitary_forward(*args))
        assert binding.last_kernel() == binding.KERNEL_LDS
        y_r = host(binding.givens_forward(dev(theta), dev(x)))
    finally:
        binding.set_kernel(binding.KERNEL_AUTO)
    assert np.abs(y_c.imag).max() == 0.0
    assert V.rel_fro(y_c.real, y_r) <= 2e-6
    assert np.abs(y_car.imag).max() <= 1e-6 * np.abs(y_r).max()   # multiples of pi are not exact in float64
    assert V.rel_fro(y_car.real, y_r) <= 4e-6


# Carousel family of the unitary extension: n a multiple of 16 from 128 to 4096.  Shapes: one lane group exactly
# (128, 256), idle lanes in the last wavefront (272), odd B (16-byte loads off, ragged last strip), several
# wavefronts (1024, 2048), a batch wide enough for the widest strips and for persistent workgroups of the
# reverse sweep that take a second strip (256 x 4100), and batches that put the reverse sweep into its shape with
# two slots per lane and several wavefronts (1024 x 520, 2048 x 264; 256 x 4100 runs it with one wavefront); the
# largest n, where the phase pass takes two pairs per thread (4096 x 16).
@pytest.mark.parametrize("n,B,seed", [(128, 9, 441), (256, 64, 442), (272, 33, 443), (1024, 20, 444), (2048, 6, 445),
                                      (256, 4100, 446), (1024, 520, 447), (2048, 264, 448), (4096, 16, 450)])
def test_carousel_family_against_the_oracle_and_the_lds_family(n, B, seed):
    theta, phi, x, g, y = check(n, B, seed, family=binding.KERNEL_CAROUSEL)
    th_d, ph_d = dev(theta), dev(phi)
    dx_c, dth_c, dph_c = (host(t) for t in binding.givens_unitary_backward(th_d, ph_d, dev(y), dev(g)))
    binding.set_kernel(binding.KERNEL_LDS)
    try:
        y_l = host(binding.givens_unitary_forward(th_d, ph_d, dev(x)))
        assert binding.last_kernel() == binding.KERNEL_LDS
        dx_l, dth_l, dph_l = (host(t) for t in binding.givens_unitary_backward(th_d, ph_d, dev(y), dev(g)))
    finally:
        binding.set_kernel(binding.KERNEL_AUTO)
    assert V.rel_fro(y, y_l) <= 1e-5
    assert V.rel_fro(dx_c, dx_l) <= 1e-5 and V.rel_fro(dth_c, dth_l) <= 1e-4 and V.rel_fro(dph_c, dph_l) <= 1e-4
    # twice the same call: bit-identical (fixed summation order)
    again = binding.givens_unitary_backward(th_d, ph_d, dev(y), dev(g))
    assert np.array_equal(host(again[1]), dth_c) and np.array_equal(host(again[2]), dph_c)


def test_carousel_family_at_the_edges_of_the_angle_reductions():
    """theta and phi on and next to the multiples of pi/2 where the reductions modulo pi change branch, angles of many
    turns, zeros; the carried phases and the three-shear forms must reproduce the oracle there too."""
    n, B = 256, 24
    theta, phi, x, g = make(n, B, 453, np.float32, np.complex64)
    pi = np.float32(np.pi)
    special = np.array([pi / 2, -pi / 2, np.nextafter(pi / 2, np.float32(4)), np.nextafter(-pi / 2, np.float32(-4)),
                        pi, -pi, np.float32(1.5) * pi, np.float32(-1.5) * pi, np.float32(3) * pi,
                        np.float32(100.25) * pi, np.float32(-999.5) * pi, np.float32(12345.678), np.float32(-9.9e5),
                        np.float32(0), np.float32(1e-30), np.float32(0.25) * pi, np.float32(-0.75) * pi], dtype=np.float32)
    rng = np.random.default_rng(454)
    for arr in (theta, phi):
        where = rng.choice(arr.size, size=16 * special.size, replace=False)
        arr[where] = np.tile(special, 16)
    th_d, ph_d = dev(theta), dev(phi)
    y_d = binding.givens_unitary_forward(th_d, ph_d, dev(x))
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    want_y = V.forward_blocks(theta, phi, x)
    dx_d, dth_d, dph_d = binding.givens_unitary_backward(th_d, ph_d, y_d, dev(g))
    want_dth, want_dph, want_dx, _ = V.reverse_sweep_blocks(theta, phi, want_y, g)
    errs = (V.rel_fro(host(y_d), want_y), V.rel_fro(host(dx_d), want_dx), V.rel_fro(host(dth_d), want_dth),
            V.rel_fro(host(dph_d), want_dph))
    print("[unitary]   special angles: Y %.2e dX %.2e dtheta %.2e dphi %.2e" % errs, flush=True)
    assert errs[0] <= 1e-5 and max(errs[1:]) <= 1e-4


def test_carousel_family_at_a_benchmark_size():
    """n = B = 2048, the shape bench.py --unitary is quoted on: sampled columns of Y and dX against the oracle
    (columns do not interact), all of dtheta and dphi against the LDS family, which the small cases pin."""
    n, B = 2048, 2048
    theta, phi, x, g = make(n, B, 451, np.float32, np.complex64)
    print(f"[unitary] n={n} B={B} seed=451 full batch", flush=True)
    th_d, ph_d = dev(theta), dev(phi)
    y_d = binding.givens_unitary_forward(th_d, ph_d, dev(x))
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    dx_d, dth_d, dph_d = binding.givens_unitary_backward(th_d, ph_d, y_d, dev(g))
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    cols = np.unique(np.concatenate([[0, 1, 7, 8, B - 1, B - 2], np.random.default_rng(452).integers(0, B, 26)]))
    want_y = V.forward_blocks(theta, phi, x[:, cols])
    y = host(y_d)
    err_y = V.rel_fro(y[:, cols], want_y)
    want_dx = V.reverse_sweep_blocks(theta, phi, want_y, g[:, cols])[2]
    err_dx = V.rel_fro(host(dx_d)[:, cols], want_dx)
    binding.set_kernel(binding.KERNEL_LDS)
    try:
        y_l = binding.givens_unitary_forward(th_d, ph_d, dev(x))
        _, dth_l, dph_l = binding.givens_unitary_backward(th_d, ph_d, y_d, dev(g))
        assert binding.last_kernel() == binding.KERNEL_LDS
    finally:
        binding.set_kernel(binding.KERNEL_AUTO)
    errs = (err_y, err_dx, V.rel_fro(y, host(y_l)), V.rel_fro(host(dth_d), host(dth_l)), V.rel_fro(host(dph_d), host(dph_l)))
    print("[unitary]   Y %.2e dX %.2e (sampled columns, oracle); Y %.2e dtheta %.2e dphi %.2e (LDS family)" % errs,
          flush=True)
    assert errs[0] <= 1e-5 and errs[1] <= 1e-4 and errs[2] <= 1e-5 and errs[3] <= 1e-4 and errs[4] <= 1e-4
    ny, nx = float(np.linalg.norm(y.astype(np.complex128))), float(np.linalg.norm(x.astype(np.complex128)))
    assert abs(ny - nx) <= 2e-6 * nx


def test_carousel_family_is_refused_for_shapes_it_does_not_cover():
    theta, phi, x, _ = make(130, 8, 449, np.float32, np.complex64)
    binding.set_kernel(binding.KERNEL_CAROUSEL)
    try:
        with pytest.raises(binding.GivensError):
            binding.givens_unitary_forward(dev(theta), dev(phi), dev(x))
    finally:
        binding.set_kernel(binding.KERNEL_AUTO)


def test_argument_errors():
    L = binding.lib()
    assert L.givens_unitary_forward(7, 4, None, None, None, None, None) == -1
    assert L.givens_unitary_forward(8, 0, None, None, None, None, None) == -2
    assert L.givens_unitary_forward(8, 4, None, None, None, None, None) == -3
    assert L.givens_unitary_backward(8, 4, None, None, None, None, None, None, None, None) == -3
