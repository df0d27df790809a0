import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(autouse=True)
def _forms_by_range(request):
    """GPU tests run the float carousel kernels with GIVENS_FORM_RANGE as the process default: the scaled and
    lifted rotation forms are then chosen from the angles whatever the size, so that the small shapes the oracle can
    check element by element exercise them.  (The library's own default, GIVENS_FORM_AUTO, takes the standard form
    below 1e9 updates; the full-size tests and a test of their own cover it.)"""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    from paper_2106_00003_amd import binding
    try:
        binding.lib()
    except Exception:
        yield
        return
    binding.set_rotation_form(binding.FORM_RANGE)
    yield
    binding.set_rotation_form(binding.FORM_AUTO)
