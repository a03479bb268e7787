import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


C_CLIENT = {"ran": False, "rc": None, "output": ""}


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The plain C client of the library (csrc/abi_demo.c, built by build()) is its own program.  On the GPU machines
    # a process that has initialised the GPU must not start other programs, so it is run here, before anything in
    # this process has touched the GPU (counting devices does not), and only when GPU tests were asked for; the
    # test that checks its result is tests/test_abi.py::test_c_client_of_the_library_runs.
    expr = config.getoption("-m", default="") or ""
    if "gpu" not in expr or "not gpu" in expr:
        return
    import subprocess
    demo = os.path.join(ROOT, "paper_2603_19289_amd", "abi_demo")
    try:
        import torch
        if not os.path.exists(demo) or torch.cuda.device_count() < 1:
            return
        done = subprocess.run([demo], capture_output=True, text=True, timeout=120)
        C_CLIENT.update(ran=True, rc=done.returncode, output=done.stdout[-2000:] + done.stderr[-2000:])
    except Exception as err:                                  # a time-out or a missing runtime: the test reports it
        C_CLIENT.update(ran=True, rc=-1, output=repr(err))


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
