"""GPU parity of the restricted parametrisation (Section 5) and odd n (end of Section 3) through the
C ABI, against oracle/restricted_oracle.py (small sizes) and the C oracle on the free pairs."""
import numpy as np
import pytest

from oracle import c_oracle as C
from oracle import givens_oracle as O
from oracle import restricted_oracle as R
from paper_2106_00003_amd import binding

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_Y, TOL_G, TOL_64 = 1e-5, 1e-4, 1e-12


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.set_rotation_form(binding.FORM_RANGE)
    yield
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.set_rotation_form(binding.FORM_RANGE)
    binding.release()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def make(n, m, B, seed, dtype=np.float32, scale=None):
    rng = np.random.default_rng(seed)
    count = R.num_free_angles(n, m)
    theta = rng.uniform(-np.pi, np.pi, count) if scale is None else rng.normal(0.0, scale, count)
    return (theta.astype(dtype), rng.standard_normal((n, B)).astype(dtype),
            rng.standard_normal((n, B)).astype(dtype))


def check(n, m, B, seed, dtype=np.float32, scale=None, kernel=binding.KERNEL_AUTO, expect_kernel=None,
          expect_form=None):
    theta, X, G = make(n, m, B, seed, dtype, scale)
    tol_y, tol_g = (TOL_64, TOL_64) if dtype == np.float64 else (TOL_Y, TOL_G)
    pairs = R.free_pairs(n, m)
    print(f"[restricted] n={n} m={m} B={B} seed={seed} angles={pairs.shape[0]}", flush=True)
    binding.set_kernel(kernel)
    th_d = dev(theta)
    y_d = binding.givens_forward_restricted(th_d, dev(X), m)
    if expect_kernel is not None:
        assert binding.last_kernel() == expect_kernel
    if expect_form is not None:
        assert binding.last_rotation_form() == expect_form
    want_y = C.forward_pairs(theta, X, pairs)
    assert O.rel_fro(host(y_d), want_y) <= tol_y
    dx_d, dth_d = binding.givens_backward_restricted(th_d, y_d, dev(G), m)
    want_dth, want_dx, _ = C.reverse_sweep_pairs(theta, want_y, G, pairs)
    assert O.rel_fro(host(dx_d), want_dx) <= tol_g
    assert O.rel_fro(host(dth_d), want_dth) <= tol_g
    u_d = binding.givens_build_restricted(th_d, n, m)
    want_u = C.forward_pairs(theta, None, pairs, n=n)
    assert O.rel_fro(host(u_d), want_u) <= tol_y
    return host(y_d), want_y


def test_section5_example_in_float64_against_the_definition():
    n, m, B = 8, 4, 5
    theta, X, G = make(n, m, B, 301, np.float64)
    u = R.dense_product(n, theta, m)                              # Eq. (2) over the 22 free pairs
    y_d = binding.givens_forward_restricted(dev(theta), dev(X), m)
    assert binding.last_kernel() == binding.KERNEL_LDS
    assert O.rel_fro(host(y_d), u @ X) <= TOL_64
    dx_d, dth_d = binding.givens_backward_restricted(dev(theta), y_d, dev(G), m)
    want_dth, want_dx, _ = R.reverse_sweep(theta, u @ X, G, m)
    assert O.rel_fro(host(dth_d), want_dth) <= TOL_64
    assert O.rel_fro(host(dx_d), u.T @ G) <= TOL_64
    assert O.rel_fro(host(binding.givens_build_restricted(dev(theta), n, m)), u) <= TOL_64


@pytest.mark.parametrize("n,m,B,seed", [(3, 2, 4, 311), (5, 2, 7, 312), (9, 8, 19, 313), (35, 10, 21, 314),
                                        (34, 5, 19, 315), (131, 130, 33, 316), (300, 1, 17, 317)])
def test_lds_family_restricted_and_odd(n, m, B, seed):
    check(n, m, B, seed, kernel=binding.KERNEL_LDS, expect_kernel=binding.KERNEL_LDS)


@pytest.mark.parametrize("n,m,B,seed", [(9, 4, 6, 321), (33, 32, 12, 322)])
def test_fp64_restricted_and_odd(n, m, B, seed):
    check(n, m, B, seed, dtype=np.float64)


@pytest.mark.parametrize("n,m,B,seed", [(256, 100, 40, 331), (255, 254, 37, 332), (511, 17, 64, 333),
                                        (1023, 1022, 48, 334), (2047, 1500, 72, 335), (1024, 1, 33, 336)])
def test_carousel_family_restricted_and_odd_general_angles(n, m, B, seed):
    check(n, m, B, seed, kernel=binding.KERNEL_CAROUSEL, expect_kernel=binding.KERNEL_CAROUSEL,
          expect_form=binding.FORM_LIFTED)


@pytest.mark.parametrize("n,m,B,seed", [(255, 100, 40, 341), (512, 300, 33, 342), (2047, 2046, 64, 343)])
def test_carousel_family_restricted_and_odd_small_angles_use_the_scaled_form(n, m, B, seed):
    check(n, m, B, seed, scale=0.1, kernel=binding.KERNEL_CAROUSEL, expect_kernel=binding.KERNEL_CAROUSEL,
          expect_form=binding.FORM_SCALED)


@pytest.mark.parametrize("n,m,B,seed", [(1001, 1000, 48, 345), (2049, 700, 40, 346), (4097, 512, 24, 347)])
def test_odd_sizes_that_pad_to_an_odd_slot_count_shape(n, m, B, seed):
    """1002 = 6 x 167, 2050 = 10 x 205, 4098 = 6 x 683: padded sizes with 3 or 5 slots per lane (standard form)."""
    check(n, m, B, seed, kernel=binding.KERNEL_AUTO, expect_kernel=binding.KERNEL_CAROUSEL,
          expect_form=binding.FORM_STANDARD)


def test_standard_form_and_forced_two_stage_reduction_with_a_restricted_problem():
    try:
        binding.set_rotation_form(binding.FORM_STANDARD)
        check(511, 200, 50, 351, kernel=binding.KERNEL_CAROUSEL, expect_form=binding.FORM_STANDARD)
        binding.set_rotation_form(binding.FORM_RANGE)
        binding.set_reduction(binding.REDUCTION_TWO_STAGE)
        check(255, 77, 1300, 352, kernel=binding.KERNEL_CAROUSEL)
        assert binding.last_reduction() == binding.REDUCTION_TWO_STAGE
    finally:
        binding.set_rotation_form(binding.FORM_RANGE)
        binding.set_reduction(binding.REDUCTION_AUTO)


def test_wide_batch_uses_the_gram_form_with_a_restricted_odd_problem():
    check(255, 100, 1030, 353, kernel=binding.KERNEL_CAROUSEL)
    assert binding.last_reduction() == binding.REDUCTION_GRAM
    check(511, 510, 2050, 354, scale=0.1, kernel=binding.KERNEL_CAROUSEL, expect_form=binding.FORM_SCALED)
    assert binding.last_reduction() == binding.REDUCTION_GRAM


@pytest.mark.parametrize("n,m,B,seed", [(35, 10, 200, 355), (64, 20, 300, 356), (127, 126, 260, 357), (9, 4, 3, 358)])
def test_column_family_restricted_and_odd(n, m, B, seed):
    check(n, m, B, seed, kernel=binding.KERNEL_AUTO)
    if B >= 2 * (n + n % 2):
        assert binding.last_reduction() == binding.REDUCTION_GRAM


@pytest.mark.parametrize("n,m,B,seed", [(999, 400, 40, 359), (299, 298, 65, 360), (1100, 3, 30, 361)])
def test_carousel_with_idle_lanes_restricted_and_odd(n, m, B, seed):
    check(n, m, B, seed, kernel=binding.KERNEL_AUTO, expect_kernel=binding.KERNEL_CAROUSEL)


def test_unrestricted_m_gives_the_unrestricted_entry_points_result():
    n, B = 256, 24
    theta, X, G = make(n, n - 1, B, 361)
    th_d, x_d = dev(theta), dev(X)
    a = host(binding.givens_forward_restricted(th_d, x_d, n - 1))
    b = host(binding.givens_forward(th_d, x_d))
    assert np.array_equal(a, b)


def test_switching_between_problems_rebuilds_the_pair_map():
    y1, w1 = check(255, 100, 16, 371)
    y2, w2 = check(255, 50, 16, 372)
    y3, w3 = check(255, 100, 16, 371)
    assert np.array_equal(y1, y3)
