"""Seeded sweep over 120 (n, B, m, angle distribution, kernel settings) combinations: every one is compared
with the oracle.  The shapes are drawn so that all kernel families, rotation forms and reductions come up."""
import numpy as np
import pytest

from oracle import c_oracle as C
from oracle import givens_oracle as O
from oracle import restricted_oracle as R
from paper_2106_00003_amd import binding

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    yield
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.set_rotation_form(binding.FORM_RANGE)
    binding.set_reduction(binding.REDUCTION_AUTO)
    binding.release()


def _cases():
    rng = np.random.default_rng(20210688)
    sizes = [2, 4, 10, 31, 32, 63, 64, 100, 127, 128, 130, 132, 135, 136, 200, 202, 255, 256, 300, 384, 500, 511,
             512, 640, 767, 768, 1000, 1002, 1023, 1024, 1032, 1280, 1536, 2040]
    out = []
    for idx in range(120):
        n = int(sizes[idx % len(sizes)])
        B = int(rng.choice([1, 3, 8, 17, 64, 100, 257, 600, 1500]))
        if n >= 1000:
            B = min(B, 300 if n < 2000 else 64)
        restricted = rng.random() < 0.4 and n >= 4
        m = int(rng.integers(1, n)) if restricted else n - 1
        if n % 2 and not restricted:
            m = n - 1
        dist = ["uniform", "small", "huge"][int(rng.integers(0, 3))]
        form = [binding.FORM_RANGE, binding.FORM_RANGE, binding.FORM_STANDARD, binding.FORM_LIFTED][int(rng.integers(0, 4))]
        red = [binding.REDUCTION_AUTO, binding.REDUCTION_TWO_STAGE, binding.REDUCTION_TWO_STAGE,
               binding.REDUCTION_GRAM][int(rng.integers(0, 4))]
        out.append((idx, n, B, m, dist, form, red))
    return out


@pytest.mark.parametrize("idx,n,B,m,dist,form,red", _cases())
def test_random_configuration_matches_the_oracle(idx, n, B, m, dist, form, red):
    rng = np.random.default_rng(7000 + idx)
    pairs = R.free_pairs(n, m)
    count = pairs.shape[0]
    if dist == "uniform":
        theta = rng.uniform(-np.pi, np.pi, count)
    elif dist == "small":
        theta = rng.normal(0.0, 0.1, count)
    else:
        theta = rng.uniform(-40.0, 40.0, count)
    theta = theta.astype(np.float32)
    X = rng.standard_normal((n, B)).astype(np.float32)
    G = rng.standard_normal((n, B)).astype(np.float32)
    print(f"[random] case {idx}: n={n} B={B} m={m} angles={dist} form={form} reduction={red}", flush=True)
    binding.set_kernel(binding.KERNEL_AUTO)
    binding.set_rotation_form(form)
    binding.set_reduction(red)
    th_d = torch.from_numpy(theta).cuda()
    y_d = binding.givens_forward_restricted(th_d, torch.from_numpy(X).cuda(), m)
    dx_d, dth_d = binding.givens_backward_restricted(th_d, y_d, torch.from_numpy(G).cuda(), m)
    torch.cuda.synchronize()
    want_y = C.forward_pairs(theta, X, pairs)
    want_dth, want_dx, _ = C.reverse_sweep_pairs(theta, want_y, G, pairs)
    assert O.rel_fro(y_d.cpu().numpy(), want_y) <= 1e-5
    assert O.rel_fro(dx_d.cpu().numpy(), want_dx) <= 1e-4
    if count:
        assert O.rel_fro(dth_d.cpu().numpy(), want_dth) <= 1e-4
