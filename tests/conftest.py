import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # A gpu-marked test must never silently pass without a device.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


# Every GPU test that is not one of the full-size workloads runs three times: with the library's
# own choice between its one-pass and two-phase kernels, and with either kind forced where it
# applies (CMN_STEP_KERNEL is read when a plan is created).  Both kinds must give the oracle's bits.
def pytest_generate_tests(metafunc):
    if "step_kernel_mode" in metafunc.fixturenames:
        on_gpu = metafunc.definition.get_closest_marker("gpu") is not None
        small = "full_size" not in metafunc.function.__name__
        modes = ["auto", "two_phase", "stream"] if on_gpu and small else ["auto"]
        metafunc.parametrize("step_kernel_mode", modes, indirect=True)


@pytest.fixture(autouse=True)
def step_kernel_mode(request, monkeypatch):
    mode = getattr(request, "param", "auto")
    if mode != "auto":
        monkeypatch.setenv("CMN_STEP_KERNEL", mode)
    return mode
