"""Host-side checks of the C-ABI library: it loads, exports what the header declares, its
schedule is bit-exact against the oracle, and argument errors come back as codes.
No GPU work is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import givens_oracle as O
from paper_2106_00003_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "givens_rr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int|int64_t|char)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    declared = _declared_functions()
    assert "givens_forward" in declared and "rr_schedule" in declared and len(declared) >= 14
    for name in declared:
        assert hasattr(L, name), f"{name} is declared in givens_rr.h but not exported"
    assert sorted(binding.EXPORTS) == declared


@pytest.mark.parametrize("n", [2, 4, 6, 8, 10, 16, 62, 256, 1024])
def test_rr_schedule_is_bit_exact_against_the_oracle(n):
    got = binding.rr_schedule(n)
    assert got.dtype == np.int32 and got.shape == (n - 1, n // 2, 2)
    if n <= 256:
        want = O.circle_method_schedule(n)
    else:
        from oracle import c_oracle
        want = c_oracle.schedule(n)
    assert np.array_equal(got, want)


def test_rr_schedule_n6_matches_the_papers_worked_example():
    got = binding.rr_schedule(6).tolist()
    assert got == [[[0, 5], [1, 4], [2, 3]], [[0, 4], [3, 5], [1, 2]], [[0, 3], [2, 4], [1, 5]],
                   [[0, 2], [1, 3], [4, 5]], [[0, 1], [2, 5], [3, 4]]]


def test_rr_schedule_full_size_properties():
    n = 4096
    s = binding.rr_schedule(n)
    flat = np.sort(s.reshape(n - 1, n), axis=1)
    assert np.array_equal(flat, np.broadcast_to(np.arange(n), (n - 1, n)))
    key = s[:, :, 0].astype(np.int64) * n + s[:, :, 1]
    assert np.unique(key).size == n * (n - 1) // 2
    assert np.all(s[:, :, 0] < s[:, :, 1])


def test_argument_errors_are_codes_not_crashes():
    L = binding.lib()
    buf = (ctypes.c_int32 * 64)()
    assert L.rr_schedule(3, buf) == -1
    assert L.rr_schedule(0, buf) == -1
    assert L.rr_schedule(4, None) == -3
    one = ctypes.c_void_p(16)      # never dereferenced: the checks below fail first
    assert L.givens_forward(5, 4, one, one, one, None) == -1
    assert L.givens_forward(4, 0, one, one, one, None) == -2
    assert L.givens_forward(4, 4, None, one, one, None) == -3
    assert L.givens_forward(4, 4, one, None, one, None) == -3
    assert L.givens_build(7, one, one, None) == -1
    assert L.givens_build(8, one, None, None) == -3
    assert L.givens_backward(4, 4, one, one, one, one, None, None) == -3
    assert L.givens_backward(4, -1, one, one, one, one, one, None) == -2
    assert L.givens_backward_f64(2, 1, one, one, one, one, one, None) in (-6, -4)  # dX aliases Y
    assert L.givens_set_kernel(99) == -5
    assert b"even" in L.givens_error_string(-1)
    with pytest.raises(binding.GivensError):
        binding.rr_schedule(7)


# ---------------------------------------------------------------- restricted parametrisation, odd n
@pytest.mark.parametrize("n,m", [(8, 4), (8, 7), (6, 1), (3, 1), (3, 2), (5, 4), (9, 3), (64, 20), (255, 254), (257, 100)])
def test_restricted_schedule_is_bit_exact_against_the_oracle(n, m):
    from oracle import restricted_oracle as R
    want = R.free_pairs(n, m)
    got = binding.rr_schedule_restricted(n, m)
    assert got.dtype == np.int32 and got.shape == want.shape
    assert np.array_equal(got, want)
    assert binding.num_angles(n, m) == R.num_free_angles(n, m) == want.shape[0]


def test_restricted_schedule_with_m_equal_n_minus_1_is_rr_schedule():
    for n in (2, 6, 16, 256):
        assert np.array_equal(binding.rr_schedule_restricted(n, n - 1), binding.rr_schedule(n).reshape(-1, 2))


def test_restricted_argument_errors():
    L = binding.lib()
    assert L.givens_num_angles(1, 1) == -1
    assert L.givens_num_angles(8, 0) == -7
    assert L.givens_num_angles(8, 8) == -7
    assert L.givens_num_angles(8, 4) == 22                      # the example of Section 5
    assert L.rr_schedule_restricted(8, 9, None) == -7
    assert L.rr_schedule_restricted(8, 4, None) == -3
    assert L.givens_forward_restricted(8, 0, 4, None, None, None, None) == -7
    assert L.givens_forward_restricted(1, 1, 4, None, None, None, None) == -1
    assert L.givens_forward_restricted(9, 4, 0, None, None, None, None) == -2
    assert L.givens_forward_restricted(9, 4, 4, None, None, None, None) == -3
    assert L.givens_backward_restricted(9, 4, 4, None, None, None, None, None, None) == -3
    assert b"m must" in L.givens_error_string(-7)
