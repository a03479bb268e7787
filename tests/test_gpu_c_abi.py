"""The library from plain C: `abi_demo` (built next to the library from csrc/abi_demo.c with the host C
compiler) drives every mode and the prefill step through the C ABI without Python or torch, and checks
finiteness, counter identities, run-to-run bit equality and hint mode == on-demand mode."""
import os
import subprocess

import pytest

from paper_2603_19289_amd import build

pytestmark = pytest.mark.gpu


def test_plain_c_client_runs_every_mode():
    assert os.path.exists(build.DEMO), f"{build.DEMO} is missing: run `python -m paper_2603_19289_amd.build`"
    print(f"[case] {build.DEMO}", flush=True)
    done = subprocess.run([build.DEMO], capture_output=True, text=True, timeout=120)
    print(done.stdout, done.stderr, flush=True)
    assert done.returncode == 0, done.stderr
    assert done.stdout.strip().endswith("abi demo ok")
