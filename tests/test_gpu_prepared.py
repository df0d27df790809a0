"""Prepared coefficients (givens_prepare + *_prepared), per-call options (*_ex) and calls on several streams,
through the C ABI.  The prepared calls run the same kernels on the same tables as the plain calls, so their
results must be bit-identical to those; the plain calls are compared with the oracle here as elsewhere.
"""
import numpy as np
import pytest

from oracle import c_oracle as C
from oracle import givens_oracle as O
from oracle import restricted_oracle as R
from paper_2106_00003_amd import binding, inputs, layer

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
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.set_reduction(binding.REDUCTION_AUTO)
    binding.release()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("n,B,seed,dist", [(256, 256, 601, "uniform"), (1024, 300, 602, "normal0.1"),
                                           (64, 700, 603, "uniform"), (130, 40, 604, "uniform"),
                                           (512, 2100, 605, "uniform"), (2048, 96, 606, "normal0.1")])
def test_prepared_calls_equal_the_plain_calls_and_the_oracle(n, B, seed, dist):
    data = inputs.make_custom(n, B, seed=seed, theta_dist=dist)
    th, X, G = data["theta"], data["X"], data["G"]
    print(f"[prepared] n={n} B={B} seed={seed} {dist}", flush=True)
    th_d, x_d, g_d = dev(th), dev(X), dev(G)
    y_ref = binding.givens_forward(th_d, x_d)
    family, form = binding.last_kernel(), binding.last_rotation_form()
    dx_ref, dth_ref = binding.givens_backward(th_d, y_ref, g_d)
    reduction = binding.last_reduction()
    u_ref = binding.givens_build(th_d, n)
    torch.cuda.synchronize()

    wide = binding.PREPARE_BACKWARD_WIDE if B >= 2 * n else binding.PREPARE_BACKWARD
    token = binding.givens_prepare(th_d, n, directions=binding.PREPARE_FORWARD | wide)
    y = binding.givens_forward_prepared(token, x_d)
    assert binding.last_kernel() == family and binding.last_rotation_form() == form
    dx, dth = binding.givens_backward_prepared(token, y, g_d, th_d.numel())
    assert binding.last_reduction() == reduction
    u = binding.givens_build_prepared(token, n, th_d.device)
    # the same token serves again: nothing above replaced the tables
    y2 = binding.givens_forward_prepared(token, x_d)
    _, dth2 = binding.givens_backward_prepared(token, y, g_d, th_d.numel(), want_dx=False)
    torch.cuda.synchronize()
    for got, ref in ((y, y_ref), (dx, dx_ref), (dth, dth_ref), (u, u_ref), (y2, y_ref), (dth2, dth_ref)):
        assert torch.equal(got, ref)

    want_y = C.forward(th, X)
    want_dth, want_dx, _ = C.reverse_sweep(th, want_y, G)
    assert O.rel_fro(y.cpu().numpy(), want_y) <= TOL_Y
    assert O.rel_fro(dx.cpu().numpy(), want_dx) <= TOL_G
    assert O.rel_fro(dth.cpu().numpy(), want_dth) <= TOL_G


def test_prepared_backward_without_the_wide_tables_runs_the_two_stage_sweep():
    n, B = 256, 1100
    data = inputs.make_custom(n, B, seed=607)
    th_d, x_d, g_d = dev(data["theta"]), dev(data["X"]), dev(data["G"])
    token = binding.givens_prepare(th_d, n)              # forward + backward, no tables for the Gram form's dX sweep
    y = binding.givens_forward_prepared(token, x_d)
    dx, dth = binding.givens_backward_prepared(token, y, g_d, th_d.numel())
    assert binding.last_reduction() == binding.REDUCTION_TWO_STAGE
    want_y = C.forward(data["theta"], data["X"])
    want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
    assert O.rel_fro(dx.cpu().numpy(), want_dx) <= TOL_G
    assert O.rel_fro(dth.cpu().numpy(), want_dth) <= TOL_G
    try:
        binding.set_reduction(binding.REDUCTION_GRAM)
        with pytest.raises(binding.GivensError) as info:
            binding.givens_backward_prepared(token, y, g_d, th_d.numel())
        assert info.value.code == binding.ERR_STALE
    finally:
        binding.set_reduction(binding.REDUCTION_AUTO)


def test_prepared_restricted_and_odd():
    n, m, B = 255, 100, 70
    data = inputs.make_restricted(n, m, B, seed=611)
    th_d, x_d, g_d = dev(data["theta"]), dev(data["X"]), dev(data["G"])
    y_ref = binding.givens_forward_restricted(th_d, x_d, m)
    dx_ref, dth_ref = binding.givens_backward_restricted(th_d, y_ref, g_d, m)
    token = binding.givens_prepare(th_d, n, m)
    y = binding.givens_forward_prepared(token, x_d)
    dx, dth = binding.givens_backward_prepared(token, y, g_d, th_d.numel())
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref) and torch.equal(dx, dx_ref) and torch.equal(dth, dth_ref)
    pairs = R.free_pairs(n, m)
    assert O.rel_fro(y.cpu().numpy(), C.forward_pairs(data["theta"], data["X"], pairs)) <= TOL_Y


def test_a_token_goes_stale_when_its_tables_are_replaced():
    n, B = 256, 64
    a, b = inputs.make_custom(n, B, seed=621), inputs.make_custom(n, B, seed=622)
    tha, thb, x_d, g_d = dev(a["theta"]), dev(b["theta"]), dev(a["X"]), dev(a["G"])
    token = binding.givens_prepare(tha, n)
    ya = binding.givens_forward_prepared(token, x_d)
    binding.givens_forward(thb, x_d)                       # replaces the forward set of this stream's workspace
    with pytest.raises(binding.GivensError) as info:
        binding.givens_forward_prepared(token, x_d)
    assert info.value.code == binding.ERR_STALE
    dxa, dtha = binding.givens_backward_prepared(token, ya, g_d, tha.numel())   # the reverse set is still there
    dx_ref, dth_ref = binding.givens_backward(tha, ya, g_d)                     # ... and this replaces it
    assert torch.equal(dxa, dx_ref) and torch.equal(dtha, dth_ref)
    with pytest.raises(binding.GivensError) as info:
        binding.givens_backward_prepared(token, ya, g_d, tha.numel())
    assert info.value.code == binding.ERR_STALE
    # a token of one stream is not known on another
    token = binding.givens_prepare(tha, n)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with pytest.raises(binding.GivensError) as info:
            binding.givens_forward_prepared(token, x_d)
        assert info.value.code == binding.ERR_STALE
    # forward only: the backward call has nothing to run on
    token = binding.givens_prepare(tha, n, directions=binding.PREPARE_FORWARD)
    binding.givens_forward_prepared(token, x_d)
    with pytest.raises(binding.GivensError) as info:
        binding.givens_backward_prepared(token, ya, g_d, tha.numel())
    assert info.value.code == binding.ERR_STALE
    # a forced family other than the one prepared for
    token = binding.givens_prepare(tha, n)
    try:
        binding.set_kernel(binding.KERNEL_LDS)
        with pytest.raises(binding.GivensError) as info:
            binding.givens_forward_prepared(token, x_d)
        assert info.value.code == binding.ERR_STALE
    finally:
        binding.set_kernel(binding.KERNEL_AUTO)
    torch.cuda.synchronize()


def test_layer_backward_survives_replaced_tables():
    """Two layers on one stream: the second forward replaces the first one's tables before its backward."""
    n, B = 256, 48
    torch.manual_seed(5)
    l1, l2 = layer.OrthogonalLinear(n), layer.OrthogonalLinear(n)
    x = torch.randn(n, B, device="cuda", requires_grad=True)
    g = torch.randn(n, B, device="cuda")
    out = l2(l1(x))
    out.backward(g)
    torch.cuda.synchronize()
    t1, t2 = l1.theta.detach().cpu().numpy(), l2.theta.detach().cpu().numpy()
    x_h, g_h = x.detach().cpu().numpy(), g.cpu().numpy()
    y1 = C.forward(t1, x_h)
    y2 = C.forward(t2, y1)
    dth2, dy1, _ = C.reverse_sweep(t2, y2, g_h)
    dth1, dx, _ = C.reverse_sweep(t1, y1, dy1)
    assert O.rel_fro(out.detach().cpu().numpy(), y2) <= TOL_Y
    assert O.rel_fro(l2.theta.grad.cpu().numpy(), dth2) <= TOL_G
    assert O.rel_fro(l1.theta.grad.cpu().numpy(), dth1) <= TOL_G
    assert O.rel_fro(x.grad.cpu().numpy(), dx) <= TOL_G
    # evaluation reuses one set of prepared tables until theta changes
    with torch.no_grad():
        e1 = l1(x.detach())
        e2 = l1(x.detach())
        assert torch.equal(e1, e2) and O.rel_fro(e1.cpu().numpy(), y1) <= TOL_Y
        l1.theta.mul_(0.5)
        e3 = l1(x.detach())
        assert O.rel_fro(e3.cpu().numpy(), C.forward(0.5 * t1, x_h)) <= TOL_Y


def test_per_call_options():
    n, B = 256, 700
    data = inputs.make_custom(n, B, seed=631)
    th, X, G = data["theta"], data["X"], data["G"]
    th_d, x_d, g_d = dev(th), dev(X), dev(G)
    want_y = C.forward(th, X)
    want_dth, want_dx, _ = C.reverse_sweep(th, want_y, G)
    for kernel, expect in ((binding.KERNEL_LDS, binding.KERNEL_LDS), (binding.KERNEL_CAROUSEL, binding.KERNEL_CAROUSEL)):
        for form in (binding.FORM_RANGE, binding.FORM_STANDARD):
            y = binding.givens_forward_ex(th_d, x_d, kernel=kernel, form=form)
            assert binding.last_kernel() == expect
            if expect == binding.KERNEL_CAROUSEL:
                assert binding.last_rotation_form() == (binding.FORM_LIFTED if form == binding.FORM_RANGE else binding.FORM_STANDARD)
            assert O.rel_fro(y.cpu().numpy(), want_y) <= TOL_Y
            for red in (binding.REDUCTION_TWO_STAGE, binding.REDUCTION_GRAM):
                dx, dth = binding.givens_backward_ex(th_d, y, g_d, kernel=kernel, form=form, reduction=red)
                assert binding.last_reduction() == red
                assert O.rel_fro(dx.cpu().numpy(), want_dx) <= TOL_G
                assert O.rel_fro(dth.cpu().numpy(), want_dth) <= TOL_G
    u = binding.givens_forward_ex(th_d, None, n=n, kernel=binding.KERNEL_CAROUSEL)
    assert O.rel_fro(u.cpu().numpy(), C.forward(th, None, n=n)) <= TOL_Y
    with pytest.raises(binding.GivensError):
        binding.givens_forward_ex(th_d, x_d, kernel=77)
    # the process-wide settings were never touched
    binding.givens_forward(th_d, x_d)
    assert binding.last_kernel() == binding.KERNEL_CAROUSEL


@pytest.mark.parametrize("n,B", [(1024, 512), (2560, 2056)])
def test_calls_on_two_streams_overlap_without_sharing_tables(n, B):
    """Two problems with different angles, each on a stream of its own, launched alternately without waiting:
    every result must equal what the same call gives alone.  2560 x 2056: reverse sweeps whose workgroups are
    chained (each stream has its own rows and flags; the two grids share the compute units)."""
    a, b = inputs.make_custom(n, B, seed=641, theta_dist="uniform"), inputs.make_custom(n, B, seed=642, theta_dist="normal0.1")
    tha, xa, ga = dev(a["theta"]), dev(a["X"]), dev(a["G"])
    thb, xb, gb = dev(b["theta"]), dev(b["X"]), dev(b["G"])
    ya_ref = binding.givens_forward(tha, xa)
    dxa_ref, dtha_ref = binding.givens_backward(tha, ya_ref, ga)
    yb_ref = binding.givens_forward(thb, xb)
    dxb_ref, dthb_ref = binding.givens_backward(thb, yb_ref, gb)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for rep in range(4):
        ya, yb = torch.empty_like(xa), torch.empty_like(xb)
        dxa, dxb = torch.empty_like(xa), torch.empty_like(xb)
        dtha, dthb = torch.empty_like(tha), torch.empty_like(thb)
        binding.givens_forward(tha, xa, Y=ya, stream=s1)
        binding.givens_forward(thb, xb, Y=yb, stream=s2)
        binding.givens_backward(tha, ya, ga, dX=dxa, dtheta=dtha, stream=s1)
        binding.givens_backward(thb, yb, gb, dX=dxb, dtheta=dthb, stream=s2)
        outs.append((ya, dxa, dtha, yb, dxb, dthb))
    s1.synchronize()
    s2.synchronize()
    for ya, dxa, dtha, yb, dxb, dthb in outs:
        assert torch.equal(ya, ya_ref) and torch.equal(dxa, dxa_ref) and torch.equal(dtha, dtha_ref)
        assert torch.equal(yb, yb_ref) and torch.equal(dxb, dxb_ref) and torch.equal(dthb, dthb_ref)


def test_restricted_shapes_alternate_on_one_stream():
    """Two restricted problems of different (n, m) take turns on one stream: the index map is rebuilt on the
    stream each time and every result still matches the oracle."""
    cases = [(255, 100, 40, 651), (300, 17, 33, 652), (255, 100, 40, 651), (301, 300, 21, 653)]
    todo = []
    for n, m, B, seed in cases:
        data = inputs.make_restricted(n, m, B, seed=seed)
        th_d, x_d, g_d = dev(data["theta"]), dev(data["X"]), dev(data["G"])
        y = binding.givens_forward_restricted(th_d, x_d, m)
        dx, dth = binding.givens_backward_restricted(th_d, y, g_d, m)
        todo.append((n, m, data, y, dx, dth))
    torch.cuda.synchronize()
    for n, m, data, y, dx, dth in todo:
        pairs = R.free_pairs(n, m)
        want_y = C.forward_pairs(data["theta"], data["X"], pairs)
        want_dth, want_dx, _ = C.reverse_sweep_pairs(data["theta"], want_y, data["G"], pairs)
        assert O.rel_fro(y.cpu().numpy(), want_y) <= TOL_Y
        assert O.rel_fro(dx.cpu().numpy(), want_dx) <= TOL_G
        assert O.rel_fro(dth.cpu().numpy(), want_dth) <= TOL_G


def test_sizes_no_kernel_family_takes_are_rejected_before_allocation():
    before = torch.cuda.mem_get_info()[0]
    th = torch.zeros(8, device="cuda")
    x = torch.zeros(8, device="cuda")
    rc = binding.lib().givens_forward_restricted(40001, 3, 1, th.data_ptr(), x.data_ptr(), x.data_ptr(), None)
    assert rc == -5
    assert abs(torch.cuda.mem_get_info()[0] - before) < (64 << 20)


def test_batch_hint_lets_prepare_follow_the_default_form_rule():
    """givens_prepare_ex with the batch: GIVENS_FORM_AUTO prepares the standard form for a short sweep and the form
    the angles allow for a long one; without the hint it always prepares the latter.  Results against the oracle."""
    from oracle import c_oracle as C
    from oracle import givens_oracle as O
    binding.set_rotation_form(binding.FORM_AUTO)
    try:
        for n, B, want in ((256, 64, binding.FORM_STANDARD), (2048, 520, binding.FORM_SCALED)):
            data = inputs.make_custom(n, B, seed=900 + n, theta_dist="normal0.1")
            th_d = torch.from_numpy(data["theta"]).cuda()
            x_d, g_d = torch.from_numpy(data["X"]).cuda(), torch.from_numpy(data["G"]).cuda()
            tok = binding.givens_prepare(th_d, n, None, binding.PREPARE_FORWARD | binding.PREPARE_BACKWARD, batch=B)
            y_d = binding.givens_forward_prepared(tok, x_d)
            assert binding.last_rotation_form() == want
            dx_d, dth_d = binding.givens_backward_prepared(tok, y_d, g_d, data["theta"].size)
            assert binding.last_rotation_form() == want
            want_y = C.forward(data["theta"], data["X"])
            want_dth, want_dx, _ = C.reverse_sweep(data["theta"], want_y, data["G"])
            assert O.rel_fro(y_d.cpu().numpy(), want_y) <= 1e-5
            assert O.rel_fro(dx_d.cpu().numpy(), want_dx) <= 1e-4
            assert O.rel_fro(dth_d.cpu().numpy(), want_dth) <= 1e-4
        data = inputs.make_custom(256, 64, seed=1156, theta_dist="normal0.1")
        tok = binding.givens_prepare(torch.from_numpy(data["theta"]).cuda(), 256, None, binding.PREPARE_FORWARD)
        binding.givens_forward_prepared(tok, torch.from_numpy(data["X"]).cuda())
        assert binding.last_rotation_form() == binding.FORM_SCALED
    finally:
        binding.set_rotation_form(binding.FORM_RANGE)
