"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Tolerances (relative Frobenius error against the oracle):
    Y, U          <= 1e-5   (fp32 kernels)
    dtheta, dX    <= 1e-4   (fp32 kernels)
    everything    <= 1e-12  (fp64 kernels)
The schedule is compared bit for bit in tests/test_library_host.py.
"""
import math

import numpy as np
import pytest

from oracle import c_oracle as C
from oracle import givens_oracle as O
from paper_2106_00003_amd import binding, inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_Y, TOL_G, TOL_64 = 1e-5, 1e-4, 1e-12


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()          # fails loudly if the library is not built
    yield
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.release()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def check_forward_backward(theta, X, G, kernel, tol_y, tol_g, expect_kernel=None):
    """Full comparison against the oracle (sizes the oracle finishes in seconds)."""
    n, B = X.shape
    binding.set_kernel(kernel)
    th_d, x_d, g_d = dev(theta), dev(X), dev(G)
    y_d = binding.givens_forward(th_d, x_d)
    if expect_kernel is not None:
        assert binding.last_kernel() == expect_kernel
    want_y = C.forward(theta, X)
    err_y = O.rel_fro(host(y_d), want_y)
    assert err_y <= tol_y, f"Y: {err_y}"
    # backward from the library's own forward output
    dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
    want_dth, want_dx, _ = C.reverse_sweep(theta, want_y, G)
    err_dx = O.rel_fro(host(dx_d), want_dx)
    err_dth = O.rel_fro(host(dth_d), want_dth)
    assert err_dx <= tol_g, f"dX: {err_dx}"
    assert err_dth <= tol_g, f"dtheta: {err_dth}"
    return err_y, err_dx, err_dth


# ---------------------------------------------------------------- config 1 (fp64)
def test_config1_fp64_forward_build_backward():
    data = inputs.make_inputs(1)
    th, X, G = data["theta"], data["X"], data["G"]
    check_forward_backward(th, X, G, binding.KERNEL_AUTO, TOL_64, TOL_64, binding.KERNEL_LDS)
    # against the explicit product of Givens matrices and per-angle central differences
    u = O.dense_product(8, th)
    u_d = binding.givens_build(dev(th), 8)
    assert O.rel_fro(host(u_d), u) <= TOL_64
    y_d = binding.givens_forward(dev(th), dev(X))
    assert O.rel_fro(host(y_d), u @ X) <= TOL_64
    _, dth_d = binding.givens_backward(dev(th), y_d, dev(G))
    fd = O.finite_difference_grad_theta(th, X, G, forward=lambda t: O.dense_product(8, t) @ X)
    assert O.rel_fro(host(dth_d), fd) <= 1e-7


# ---------------------------------------------------------------- config 2
@pytest.mark.parametrize("kernel,expect", [(binding.KERNEL_LDS, binding.KERNEL_LDS),
                                           (binding.KERNEL_AUTO, binding.KERNEL_CAROUSEL)])
def test_config2_n256_forward_backward(kernel, expect):
    data = inputs.make_inputs(2)
    check_forward_backward(data["theta"], data["X"], data["G"], kernel, TOL_Y, TOL_G)
    binding.set_kernel(kernel)
    binding.givens_forward(dev(data["theta"]), dev(data["X"]))
    assert binding.last_kernel() == expect


# ---------------------------------------------------------------- config 3 (build U, X = I)
def test_config3_n1024_build_and_gradient():
    data = inputs.make_inputs(3)
    th, G = data["theta"], data["G"]
    n = 1024
    binding.set_kernel(binding.KERNEL_AUTO)
    th_d = dev(th)
    u_d = binding.givens_build(th_d, n)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    want_u = C.forward(th, None, n=n)
    u = host(u_d)
    assert O.rel_fro(u, want_u) <= TOL_Y
    assert O.rel_fro(u.astype(np.float64).T @ u.astype(np.float64), np.eye(n)) <= 1e-5
    # gradient of L = sum(G * U): Algorithm 3 with Gamma = G, and the reverse sweep, in the oracle
    want_dth = C.grad_theta_alg3(th, want_u, G)
    _, dth_d = binding.givens_backward(th_d, u_d, dev(G), want_dx=False)
    assert O.rel_fro(host(dth_d), want_dth) <= TOL_G
    # same build through the LDS family
    binding.set_kernel(binding.KERNEL_LDS)
    u2_d = binding.givens_build(th_d, n)
    assert binding.last_kernel() == binding.KERNEL_LDS
    assert O.rel_fro(host(u2_d), want_u) <= TOL_Y


# ---------------------------------------------------------------- ragged / odd shapes, both families
@pytest.mark.parametrize("n,B,seed", [(2, 1, 1), (4, 3, 2), (6, 5, 3), (34, 19, 4), (130, 77, 5), (300, 41, 6)])
def test_lds_family_small_and_ragged_shapes(n, B, seed):
    data = inputs.make_custom(n, B, seed=seed)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_LDS, TOL_Y, TOL_G,
                           binding.KERNEL_LDS)


@pytest.mark.parametrize("n,B,seed", [(256, 1, 11), (256, 37, 12), (512, 100, 13), (1024, 67, 14),
                                      (2048, 130, 15), (256, 4100, 16)])
def test_carousel_family_ragged_batches(n, B, seed):
    data = inputs.make_custom(n, B, seed=seed)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G,
                           binding.KERNEL_CAROUSEL)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL      # the reverse sweep too


# ---------------------------------------------------------------- column family (n <= 128)
@pytest.mark.parametrize("n,B,seed", [(2, 5, 101), (4, 3, 102), (6, 300, 103), (8, 1, 104), (34, 77, 105),
                                      (64, 1000, 106), (100, 513, 107), (126, 260, 108), (128, 300, 109)])
def test_column_family_small_n(n, B, seed):
    data = inputs.make_custom(n, B, seed=seed)
    binding.set_kernel(binding.KERNEL_AUTO)
    th_d = dev(data["theta"])
    y_d = binding.givens_forward(th_d, dev(data["X"]))
    assert binding.last_kernel() == binding.KERNEL_COLUMN
    want_y = C.forward(data["theta"], data["X"])
    assert O.rel_fro(host(y_d), want_y) <= TOL_Y
    u_d = binding.givens_build(th_d, n)
    assert binding.last_kernel() == binding.KERNEL_COLUMN
    assert O.rel_fro(host(u_d), C.forward(data["theta"], None, n=n)) <= TOL_Y
    dx_d, dth_d = binding.givens_backward(th_d, y_d, dev(data["G"]))
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
    if B >= 2 * n:                                            # Gram form: GEMM, sweep on C, mirrored column kernel
        assert binding.last_kernel() == binding.KERNEL_COLUMN
        assert binding.last_reduction() == binding.REDUCTION_GRAM
    else:
        assert binding.last_kernel() == binding.KERNEL_LDS
    assert O.rel_fro(host(dx_d), want_dx) <= TOL_G
    assert O.rel_fro(host(dth_d), want_dth) <= TOL_G
    # the same through the LDS family, and in place through the column family
    binding.set_kernel(binding.KERNEL_LDS)
    y2 = host(binding.givens_forward(th_d, dev(data["X"])))
    binding.set_kernel(binding.KERNEL_COLUMN)
    buf = dev(data["X"])
    binding.givens_forward(th_d, buf, Y=buf)
    assert np.array_equal(host(buf), host(y_d))
    assert O.rel_fro(y2, host(y_d)) <= 2e-6
    binding.set_kernel(binding.KERNEL_AUTO)


def test_column_family_rejects_large_n_when_forced():
    data = inputs.make_custom(130, 8, seed=110)
    binding.set_kernel(binding.KERNEL_COLUMN)
    with pytest.raises(binding.GivensError) as err:
        binding.givens_forward(dev(data["theta"]), dev(data["X"]))
    assert err.value.code == -5
    binding.set_kernel(binding.KERNEL_AUTO)


@pytest.mark.parametrize("n,B,seed,dist", [(768, 70, 17, "uniform"), (1280, 45, 18, "normal0.1"),
                                           (1536, 130, 19, "uniform"), (1792, 33, 20, "uniform"),
                                           (2560, 64, 22, "normal0.1"), (3072, 40, 23, "uniform"),
                                           (3584, 24, 24, "uniform")])
def test_carousel_family_sizes_with_3_5_6_7_wavefronts(n, B, seed, dist):
    """n = 128 * WAVES * M with a wavefront count that is not a power of two."""
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G,
                           binding.KERNEL_CAROUSEL)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL


@pytest.mark.parametrize("n,B,seed,dist,red", [
    (132, 50, 131, "uniform", "two_stage"), (136, 300, 132, "normal0.1", "gram"), (200, 70, 133, "uniform", "two_stage"),
    (300, 41, 134, "uniform", "two_stage"), (1000, 64, 135, "normal0.1", "two_stage"),
    (1008, 33, 136, "uniform", "gram"), (1040, 40, 137, "uniform", "two_stage"),
    (2044, 24, 138, "uniform", "two_stage"), (2600, 20, 139, "normal0.1", "gram"), (4088, 12, 140, "uniform", "two_stage")])
def test_carousel_family_with_partly_filled_last_wavefront(n, B, seed, dist, red):
    """n = 2 M L with a lane count L that is not a multiple of 64: the spare lanes of the last wavefront idle."""
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    mode = {"two_stage": binding.REDUCTION_TWO_STAGE, "gram": binding.REDUCTION_GRAM}[red]
    try:
        binding.set_reduction(mode)
        check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                               binding.KERNEL_CAROUSEL)
        assert binding.last_kernel() == binding.KERNEL_CAROUSEL
        assert binding.last_reduction() == mode
    finally:
        binding.set_reduction(binding.REDUCTION_AUTO)
    u_d = binding.givens_build(dev(data["theta"]), n)
    assert O.rel_fro(host(u_d), C.forward(data["theta"], None, n=n)) <= TOL_Y
    binding.release()


@pytest.mark.parametrize("n,B,seed,dist", [(5120, 16, 25, "uniform"), (6144, 12, 26, "uniform"),
                                           (7168, 9, 27, "normal0.1"), (8176, 8, 28, "uniform"),
                                           (4112, 8, 29, "uniform"), (8192, 8, 30, "normal0.1"),
                                           (4112, 1040, 31, "normal0.1")])
def test_carousel_sizes_above_4096(n, B, seed, dist):
    """Multiples of 16 beyond 4096: 8 slots per lane in both sweeps (5 to 8 wavefronts, the last one partly
    filled at 4112 and 8176); 4112 x 1040 gives the reverse sweep's persistent workgroups a second strip."""
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    print(f"[parity] n={n} B={B} seed={seed} {dist}", flush=True)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                           binding.KERNEL_CAROUSEL)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL      # the reverse sweep too
    assert binding.last_reduction() == binding.REDUCTION_TWO_STAGE
    binding.release()


@pytest.mark.parametrize("n,B,seed,dist", [(2052, 24, 32, "uniform"), (4092, 12, 33, "normal0.1"),
                                           (3004, 40, 34, "uniform"), (4104, 16, 35, "uniform"),
                                           (6152, 8, 36, "normal0.1"), (8184, 8, 37, "uniform"),
                                           (2060, 2200, 38, "normal0.1")])
def test_carousel_shapes_with_more_than_512_lanes(n, B, seed, dist):
    """Multiples of 4 beyond 2048 that are not multiples of 8 (2 slots per lane) and multiples of 8 beyond 4096 that
    are not multiples of 16 (4 slots per lane): 513 to 1024 lanes, 10 to 16 wavefronts, both sweeps; 2060 x 2200
    gives the reverse sweep's persistent workgroups (one per compute unit here) a second strip."""
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    print(f"[parity] n={n} B={B} seed={seed} {dist}", flush=True)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                           binding.KERNEL_CAROUSEL)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL      # the reverse sweep too
    binding.release()


@pytest.mark.parametrize("n,B,seed,dist", [(210, 33, 41, "uniform"), (1002, 70, 42, "uniform"),
                                           (1010, 2100, 43, "normal0.1"), (2114, 40, 44, "uniform"),
                                           (2050, 600, 45, "uniform"), (4098, 16, 46, "normal0.1"),
                                           (6126, 8, 47, "uniform"), (8400, 8, 48, "uniform"),
                                           (9010, 6, 49, "normal0.1"), (4100, 24, 50, "uniform")])
def test_carousel_shapes_with_an_odd_number_of_slots_per_lane(n, B, seed, dist):
    """Even n that no shape with 2, 4 or 8 slots per lane covers (n = 2 mod 4, and multiples of 4 or 8 too large
    for 1024 lanes), with a factor 7, 5 or 3 in n / 2: 7 slots (210, 2114, 8400), 5 (1010, 2050, 4100, 9010) and
    3 (1002, 4098, 6126) per lane, 1 to 16 wavefronts; standard rotation form whatever the angles, both sweeps;
    1010 x 2100 takes the Gram form, 2050 x 600 gives persistent workgroups a second strip."""
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    print(f"[parity] n={n} B={B} seed={seed} {dist}", flush=True)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                           binding.KERNEL_CAROUSEL)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL      # the reverse sweep too
    assert binding.last_rotation_form() == binding.FORM_STANDARD
    binding.release()


@pytest.mark.parametrize("slots", [3, 5, 7])
def test_every_workgroup_size_of_the_odd_slot_count_shapes(slots):
    """n = 2 M L with L = 64 w - 3 lanes for every compiled number of wavefronts w (1..8, 10, 12, 14, 16): n / 2 is
    odd, so only a shape with an odd slot count applies (M itself, or another odd factor of L with fewer lanes);
    narrow batch, so the narrow strip widths are the ones that run, with a ragged last strip."""
    for w in (1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16):
        n = 2 * slots * (64 * w - 3)
        if n < 132:
            continue
        B = 3 if n > 6000 else 7
        data = inputs.make_custom(n, B, seed=7000 + n)
        print(f"[parity] slots={slots} wavefronts={w} n={n} B={B}", flush=True)
        check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                               binding.KERNEL_CAROUSEL)
        assert binding.last_kernel() == binding.KERNEL_CAROUSEL
        binding.release()


def test_every_even_size_up_to_700_matches_the_oracle_in_its_default_family():
    """All even n from 130 to 700 (carousel shapes with 8, 4, 2, 7, 5 or 3 slots per lane, LDS family where n / 2 is
    a prime), forward and reverse sweeps, B = 5."""
    families = set()
    for n in range(130, 701, 2):
        data = inputs.make_custom(n, 5, seed=9000 + n)
        if n % 50 == 0:
            print(f"[parity] n={n}", flush=True)
        check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G)
        families.add(binding.last_kernel())
    assert families == {binding.KERNEL_CAROUSEL, binding.KERNEL_LDS}
    binding.release()


@pytest.mark.parametrize("n,B,seed,dist", [(136, 5, 61, "uniform"), (200, 64, 62, "normal0.1"),
                                           (256, 256, 63, "uniform"), (256, 1030, 64, "uniform"),
                                           (256, 4100, 65, "normal0.1"), (384, 300, 66, "uniform"),
                                           (512, 1024, 67, "uniform"), (512, 2500, 68, "normal0.1"),
                                           (768, 40, 69, "uniform"), (768, 600, 70, "uniform"),
                                           (1024, 512, 71, "normal0.1"), (1024, 2048, 72, "uniform"),
                                           (1024, 2052, 73, "uniform"), (140, 9, 74, "uniform"),
                                           (256, 16400, 75, "uniform"), (1024, 8200, 76, "normal0.1")])
def test_one_wavefront_shapes_with_the_exchange_inside_the_wavefront(n, B, seed, dist):
    """Multiples of 8 up to 1024 with small and medium batches run one wavefront per strip and move the slots with
    wavefront shifts: 2, 4 and 8 slots per lane, fewer than 64 lanes (136, 200, 384, 768), strips of 1, 2, 4 and 8
    columns on both sides of the batch sizes where the width changes, ragged last strips, all three rotation
    forms (the angles decide); 140 is not a multiple of 8 and keeps the LDS exchange."""
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    print(f"[parity] n={n} B={B} seed={seed} {dist}", flush=True)
    binding.set_reduction(binding.REDUCTION_TWO_STAGE)       # the reverse sweep over all B columns
    try:
        check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                               binding.KERNEL_CAROUSEL)
        assert binding.last_kernel() == binding.KERNEL_CAROUSEL
        binding.set_rotation_form(binding.FORM_STANDARD)
        check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G)
    finally:
        binding.set_rotation_form(binding.FORM_RANGE)
        binding.set_reduction(binding.REDUCTION_AUTO)
    binding.release()


@pytest.mark.parametrize("n,B,seed,dist", [(2112, 2056, 81, "uniform"), (2560, 4100, 82, "normal0.1"),
                                           (3072, 2048, 83, "uniform"), (3584, 4104, 84, "normal0.1"),
                                           (4096, 2056, 85, "uniform"), (2048, 4100, 86, "uniform")])
def test_reverse_sweep_with_chained_rows_of_partial_sums(n, B, seed, dist):
    """Large two-stage reverse sweeps (n = 2112 .. 4096, a multiple of 64: workgroups of 5 to 8 wavefronts, one per
    compute unit) link their 256 persistent workgroups into chains that share rows of partial sums: exactly one pass
    (3072 x 2048), one pass plus a ragged second one (257 strips), two passes plus a ragged third (513 strips:
    2560 x 4100, 3584 x 4104); 2048 x 4100 has 4 wavefronts per workgroup and keeps separate rows.  Every component
    against the oracle, and twice: the result must be the same bit for bit."""
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    print(f"[parity] n={n} B={B} seed={seed} {dist}", flush=True)
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.set_reduction(binding.REDUCTION_TWO_STAGE)
    try:
        th_d, g_d = dev(data["theta"]), dev(data["G"])
        y_d = binding.givens_forward(th_d, dev(data["X"]))
        dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
        assert binding.last_kernel() == binding.KERNEL_CAROUSEL
        assert binding.last_reduction() == binding.REDUCTION_TWO_STAGE
        assert binding.last_chains() == (0 if n == 2048 else 32)   # 256 workgroups in chains of 8, or separate rows
        want_y = C.forward(data["theta"], data["X"])
        want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
        got_dth = host(dth_d)
        assert np.isfinite(got_dth).all()
        assert O.rel_fro(host(dx_d), want_dx) <= TOL_G
        assert O.rel_fro(got_dth, want_dth) <= TOL_G
        assert float(np.abs(got_dth - want_dth).max()) <= 1e-3 * float(np.abs(want_dth).max())
        dx2_d, dth2_d = binding.givens_backward(th_d, y_d, g_d)
        assert np.array_equal(host(dth2_d), got_dth) and np.array_equal(host(dx2_d), host(dx_d))
    finally:
        binding.set_reduction(binding.REDUCTION_AUTO)
    binding.release()


def test_sizes_whose_half_is_a_prime_stay_in_the_lds_family():
    """n = 2 p with p prime has no carousel shape (the slot count must divide n / 2)."""
    data = inputs.make_custom(1006, 40, seed=39)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G, binding.KERNEL_LDS)
    assert binding.last_kernel() == binding.KERNEL_LDS


# ---------------------------------------------------------------- scaled rotation form (near-identity angles)
@pytest.mark.parametrize("n,B,seed", [(256, 64, 51), (512, 100, 52), (1024, 67, 53), (2048, 130, 54)])
def test_scaled_form_is_used_for_small_angles_and_matches_the_oracle(n, B, seed):
    data = inputs.make_custom(n, B, seed=seed, theta_dist="normal0.1")
    assert float(np.abs(data["theta"]).max()) < 0.78
    binding.set_rotation_form(binding.FORM_RANGE)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G,
                           binding.KERNEL_CAROUSEL)
    assert binding.last_rotation_form() == binding.FORM_SCALED
    try:
        binding.set_rotation_form(binding.FORM_STANDARD)
        check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G)
        assert binding.last_rotation_form() == binding.FORM_STANDARD
    finally:
        binding.set_rotation_form(binding.FORM_RANGE)


def test_default_form_follows_the_size_of_the_sweep():
    """GIVENS_FORM_AUTO: the standard form below 1e9 updates (the scaled and lifted forms' extra coefficient work
    does not pay there), the form the angles allow from there on; both against the oracle."""
    small = inputs.make_custom(256, 64, seed=55, theta_dist="normal0.1")
    large = inputs.make_custom(2048, 520, seed=56, theta_dist="normal0.1")       # 2.1e6 angles x 520 columns
    binding.set_rotation_form(binding.FORM_AUTO)
    try:
        check_forward_backward(small["theta"], small["X"], small["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                               binding.KERNEL_CAROUSEL)
        assert binding.last_rotation_form() == binding.FORM_STANDARD
        check_forward_backward(large["theta"], large["X"], large["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G,
                               binding.KERNEL_CAROUSEL)
        assert binding.last_rotation_form() == binding.FORM_SCALED
    finally:
        binding.set_rotation_form(binding.FORM_RANGE)


def test_rotation_form_switches_at_the_angle_threshold():
    n, B = 512, 48
    data = inputs.make_custom(n, B, seed=61)
    theta = (data["theta"] * np.float32(0.245)).astype(np.float32)     # uniform in about +-0.77
    assert float(np.abs(theta).max()) <= 0.78
    check_forward_backward(theta, data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G)
    assert binding.last_rotation_form() == binding.FORM_SCALED
    theta[777] = np.float32(-0.80)                                     # one angle beyond pi/4
    check_forward_backward(theta, data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G)
    assert binding.last_rotation_form() == binding.FORM_LIFTED
    theta[777] = np.float32(2.0e6)                                     # beyond the lifted form's range
    check_forward_backward(theta, data["X"], data["G"], binding.KERNEL_AUTO, TOL_Y, TOL_G)
    assert binding.last_rotation_form() == binding.FORM_STANDARD
    for bad in ("nan", "inf"):                                         # must select neither special form
        theta[777] = np.float32(bad)
        binding.givens_forward(dev(theta), dev(data["X"]))
        assert binding.last_rotation_form() == binding.FORM_STANDARD


# ---------------------------------------------------------------- lifted rotation form (general angles)
@pytest.mark.parametrize("n,B,seed", [(256, 64, 81), (512, 100, 82), (1024, 67, 83), (2048, 130, 84)])
def test_lifted_form_is_used_for_general_angles_and_matches_the_oracle(n, B, seed):
    data = inputs.make_custom(n, B, seed=seed)                         # theta uniform in [-pi, pi)
    binding.set_rotation_form(binding.FORM_RANGE)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G,
                           binding.KERNEL_CAROUSEL)
    assert binding.last_rotation_form() == binding.FORM_LIFTED
    try:
        binding.set_rotation_form(binding.FORM_STANDARD)
        check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G)
        assert binding.last_rotation_form() == binding.FORM_STANDARD
    finally:
        binding.set_rotation_form(binding.FORM_RANGE)


def test_lifted_form_at_the_edges_of_the_angle_reduction():
    """Angles on and next to the multiples of pi/2 where the reduction modulo pi changes branch, angles
    of many turns, and the lifted form forced on near-identity angles."""
    n, B = 512, 40
    data = inputs.make_custom(n, B, seed=85)
    theta = data["theta"].copy()
    pi = np.float32(np.pi)
    special = [pi / 2, -pi / 2, np.nextafter(pi / 2, np.float32(4)), np.nextafter(-pi / 2, np.float32(-4)),
               pi, -pi, np.float32(1.5) * pi, np.float32(-1.5) * pi, np.float32(3) * pi, np.float32(100.25) * pi,
               np.float32(-999.5) * pi, np.float32(12345.678), np.float32(-9.9e5), np.float32(0), np.float32(1e-30)]
    rng = np.random.default_rng(85)
    where = rng.choice(theta.size, size=8 * len(special), replace=False)
    theta[where] = np.tile(np.array(special, dtype=np.float32), 8)
    check_forward_backward(theta, data["X"], data["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G)
    assert binding.last_rotation_form() == binding.FORM_LIFTED
    small = inputs.make_custom(n, B, seed=86, theta_dist="normal0.1")
    try:
        binding.set_rotation_form(binding.FORM_LIFTED)
        check_forward_backward(small["theta"], small["X"], small["G"], binding.KERNEL_CAROUSEL, TOL_Y, TOL_G)
        assert binding.last_rotation_form() == binding.FORM_LIFTED
    finally:
        binding.set_rotation_form(binding.FORM_RANGE)


# ---------------------------------------------------------------- the two-stage reduction is reproducible
@pytest.mark.parametrize("n,B,seed,dist", [(256, 300, 71, "uniform"), (1024, 200, 72, "normal0.1"),
                                           (2048, 64, 73, "uniform")])
def test_two_stage_reduction_matches_the_oracle_and_is_bit_reproducible(n, B, seed, dist):
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    binding.set_kernel(binding.KERNEL_CAROUSEL)
    th_d, g_d = dev(data["theta"]), dev(data["G"])
    y_d = binding.givens_forward(th_d, dev(data["X"]))
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], C.forward(data["theta"], data["X"]), data["G"])
    try:
        binding.set_reduction(binding.REDUCTION_TWO_STAGE)
        dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
        assert binding.last_reduction() == binding.REDUCTION_TWO_STAGE
        first = host(dth_d)
        assert O.rel_fro(first, want_dth) <= TOL_G
        assert O.rel_fro(host(dx_d), want_dx) <= TOL_G
        _, again = binding.givens_backward(th_d, y_d, g_d)
        assert np.array_equal(host(again), first)
    finally:
        binding.set_reduction(binding.REDUCTION_AUTO)
        binding.set_kernel(binding.KERNEL_AUTO)


# ---------------------------------------------------------------- Gram-matrix form for wide batches
@pytest.mark.parametrize("n,B,seed,dist", [(256, 1100, 75, "uniform"), (512, 2100, 76, "normal0.1"),
                                           (1024, 4096, 77, "uniform")])
def test_gram_reduction_for_wide_batches_matches_the_oracle(n, B, seed, dist):
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    binding.set_kernel(binding.KERNEL_CAROUSEL)
    th_d, g_d = dev(data["theta"]), dev(data["G"])
    y_d = binding.givens_forward(th_d, dev(data["X"]))
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], C.forward(data["theta"], data["X"]), data["G"])
    try:
        binding.set_reduction(binding.REDUCTION_AUTO)                  # B >= 2 n: the Gram form is the default
        dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
        assert binding.last_reduction() == binding.REDUCTION_GRAM
        assert O.rel_fro(host(dth_d), want_dth) <= TOL_G
        assert O.rel_fro(host(dx_d), want_dx) <= TOL_G
        first = host(dth_d).copy()
        _, again = binding.givens_backward(th_d, y_d, g_d, want_dx=False)
        assert np.array_equal(host(again), first)                      # reproducible
        # dX written over G
        g_buf = dev(data["G"])
        binding.givens_backward(th_d, y_d, g_buf, dX=g_buf)
        assert O.rel_fro(host(g_buf), want_dx) <= TOL_G
        binding.set_reduction(binding.REDUCTION_TWO_STAGE)
        _, two = binding.givens_backward(th_d, y_d, g_d, want_dx=False)
        assert binding.last_reduction() == binding.REDUCTION_TWO_STAGE
        assert O.rel_fro(first, host(two)) <= 1e-5
    finally:
        binding.set_reduction(binding.REDUCTION_AUTO)
        binding.set_kernel(binding.KERNEL_AUTO)


def test_gram_reduction_can_be_forced_on_a_narrow_batch_in_both_families():
    data = inputs.make_custom(256, 40, seed=78)
    th_d, g_d = dev(data["theta"]), dev(data["G"])
    want_y = C.forward(data["theta"], data["X"])
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
    try:
        binding.set_reduction(binding.REDUCTION_GRAM)
        binding.set_kernel(binding.KERNEL_CAROUSEL)
        y_d = binding.givens_forward(th_d, dev(data["X"]))
        dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
        assert binding.last_reduction() == binding.REDUCTION_GRAM
        assert O.rel_fro(host(dth_d), want_dth) <= TOL_G and O.rel_fro(host(dx_d), want_dx) <= TOL_G
        binding.set_kernel(binding.KERNEL_LDS)
        dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
        assert binding.last_reduction() == binding.REDUCTION_GRAM and binding.last_kernel() == binding.KERNEL_LDS
        assert O.rel_fro(host(dth_d), want_dth) <= TOL_G and O.rel_fro(host(dx_d), want_dx) <= TOL_G
        # the float64 entry points keep the two-stage reduction
        d64 = inputs.make_custom(34, 19, seed=78, dtype=np.float64)
        y64 = binding.givens_forward(dev(d64["theta"]), dev(d64["X"]))
        binding.givens_backward(dev(d64["theta"]), y64, dev(d64["G"]))
        assert binding.last_reduction() == binding.REDUCTION_TWO_STAGE
    finally:
        binding.set_reduction(binding.REDUCTION_AUTO)
        binding.set_kernel(binding.KERNEL_AUTO)


@pytest.mark.parametrize("n,B,seed", [(202, 900, 111), (302, 700, 112), (1006, 2100, 113)])
def test_lds_family_wide_batches_use_the_gram_form(n, B, seed):
    data = inputs.make_custom(n, B, seed=seed)
    binding.set_kernel(binding.KERNEL_AUTO)
    th_d = dev(data["theta"])
    y_d = binding.givens_forward(th_d, dev(data["X"]))
    assert binding.last_kernel() == binding.KERNEL_LDS
    want_y = C.forward(data["theta"], data["X"])
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
    dx_d, dth_d = binding.givens_backward(th_d, y_d, dev(data["G"]))
    assert binding.last_reduction() == binding.REDUCTION_GRAM
    assert O.rel_fro(host(dx_d), want_dx) <= TOL_G
    assert O.rel_fro(host(dth_d), want_dth) <= TOL_G


def test_largest_compiled_carousel_size_n8192():
    """n = 8192 is the largest carousel shape of both sweeps; the LDS family still takes it when asked."""
    n, B = 8192, 24
    data = inputs.make_custom(n, B, seed=79)
    binding.set_kernel(binding.KERNEL_AUTO)
    th_d = dev(data["theta"])
    y_d = binding.givens_forward(th_d, dev(data["X"]))
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    want_y = C.forward(data["theta"], data["X"])
    assert O.rel_fro(host(y_d), want_y) <= TOL_Y
    dx_d, dth_d = binding.givens_backward(th_d, y_d, dev(data["G"]))
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"], want_x=False)
    assert O.rel_fro(host(dx_d), want_dx) <= TOL_G
    assert O.rel_fro(host(dth_d), want_dth) <= TOL_G
    binding.set_kernel(binding.KERNEL_LDS)
    try:
        dx_l, dth_l = binding.givens_backward(th_d, y_d, dev(data["G"]))
        assert binding.last_kernel() == binding.KERNEL_LDS
    finally:
        binding.set_kernel(binding.KERNEL_AUTO)
    assert O.rel_fro(host(dx_l), want_dx) <= TOL_G
    assert O.rel_fro(host(dth_l), want_dth) <= TOL_G
    binding.release()


def test_carousel_rejects_shapes_it_does_not_cover():
    data = inputs.make_custom(34, 8, seed=1)
    binding.set_kernel(binding.KERNEL_CAROUSEL)
    with pytest.raises(binding.GivensError) as err:
        binding.givens_forward(dev(data["theta"]), dev(data["X"]))
    assert err.value.code == -5
    binding.set_kernel(binding.KERNEL_AUTO)


def test_fp64_ragged():
    data = inputs.make_custom(34, 19, seed=21, dtype=np.float64)
    check_forward_backward(data["theta"], data["X"], data["G"], binding.KERNEL_AUTO, TOL_64, TOL_64)


@pytest.mark.parametrize("kernel", [binding.KERNEL_LDS, binding.KERNEL_AUTO])
def test_in_place_forward_and_backward(kernel):
    data = inputs.make_custom(256, 64, seed=31)
    binding.set_kernel(kernel)
    th_d = dev(data["theta"])
    buf = dev(data["X"])
    binding.givens_forward(th_d, buf, Y=buf)
    want_y = C.forward(data["theta"], data["X"])
    assert O.rel_fro(host(buf), want_y) <= TOL_Y
    g_buf = dev(data["G"])
    dx_d, dth_d = binding.givens_backward(th_d, buf, g_buf, dX=g_buf)
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
    assert O.rel_fro(host(g_buf), want_dx) <= TOL_G
    assert O.rel_fro(host(dth_d), want_dth) <= TOL_G


def test_zero_angles_and_single_angle():
    n, B = 256, 16
    data = inputs.make_custom(n, B, seed=41)
    binding.set_kernel(binding.KERNEL_AUTO)
    th = np.zeros(n * (n - 1) // 2, dtype=np.float32)
    y = host(binding.givens_forward(dev(th), dev(data["X"])))
    assert np.array_equal(y, data["X"])
    e = 12345
    th[e] = 0.625
    i, j = binding.rr_schedule(n).reshape(-1, 2)[e]
    want = data["X"].astype(np.float64).copy()
    c, s = math.cos(0.625), math.sin(0.625)
    want[i], want[j] = c * want[i] - s * want[j], s * data["X"][i].astype(np.float64) + c * want[j]
    y = host(binding.givens_forward(dev(th), dev(data["X"])))
    assert O.rel_fro(y, want) <= 1e-7


def test_upstream_equal_to_output_gives_tiny_gradient():
    data = inputs.make_inputs(2)
    binding.set_kernel(binding.KERNEL_AUTO)
    th_d = dev(data["theta"])
    y_d = binding.givens_forward(th_d, dev(data["X"]))
    dx_d, dth_d = binding.givens_backward(th_d, y_d, y_d.clone())
    # gradient of a constant: every term cancels up to rounding; dX recovers X
    scale = float(np.linalg.norm(data["X"])) ** 2
    assert float(np.max(np.abs(host(dth_d)))) <= 1e-5 * scale / 256
    assert O.rel_fro(host(dx_d), data["X"]) <= TOL_G


def test_calls_on_a_side_stream_and_event_timing():
    data = inputs.make_custom(512, 96, seed=90)
    want_y = C.forward(data["theta"], data["X"])
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
    binding.set_kernel(binding.KERNEL_AUTO)
    side = torch.cuda.Stream()
    th_d, x_d, g_d = dev(data["theta"]), dev(data["X"]), dev(data["G"])
    torch.cuda.synchronize()
    binding.set_timing(True)
    try:
        with torch.cuda.stream(side):
            y_d = binding.givens_forward(th_d, x_d)                # the binding passes torch's current stream
            t_fwd = binding.last_timing()
            dx_d, dth_d = binding.givens_backward(th_d, y_d, g_d)
            t_bwd = binding.last_timing()
        side.synchronize()
    finally:
        binding.set_timing(False)
    assert O.rel_fro(y_d.cpu().numpy(), want_y) <= TOL_Y
    assert O.rel_fro(dx_d.cpu().numpy(), want_dx) <= TOL_G
    assert O.rel_fro(dth_d.cpu().numpy(), want_dth) <= TOL_G
    assert t_fwd[0] > 0 and t_fwd[1] > 0 and t_fwd[2] == 0          # coefficient kernels, sweep, no reduction
    assert t_bwd[0] > 0 and t_bwd[1] > 0 and t_bwd[2] > 0
    with pytest.raises(binding.GivensError):
        binding.givens_forward(th_d, x_d)
        binding.last_timing()                                       # timing was off for that call


@pytest.mark.parametrize("n,B,seed,dtype", [(8, 5, 121, np.float64), (34, 19, 122, np.float64), (64, 300, 123, np.float32),
                                            (200, 90, 124, np.float32), (256, 130, 125, np.float32),
                                            (1536, 40, 126, np.float32), (2048, 64, 127, np.float32)])
def test_transposed_forward_is_the_inverse_transform(n, B, seed, dtype):
    data = inputs.make_custom(n, B, seed=seed, dtype=dtype)
    tol = TOL_64 if dtype == np.float64 else TOL_Y
    binding.set_kernel(binding.KERNEL_AUTO)
    th_d = dev(data["theta"])
    z_d = binding.givens_forward_transposed(th_d, dev(data["G"]))
    assert O.rel_fro(host(z_d), C.grad_operand(data["theta"], data["G"])) <= tol        # U^T G by the oracle
    back = binding.givens_forward(th_d, z_d)
    assert O.rel_fro(host(back), data["G"]) <= 3 * tol                                    # U U^T G = G
