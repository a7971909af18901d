"""The library driven from a plain host program through include/mux.h alone (no Python binding,
no torch): paper_2404_02015_amd/examples/c_abi_demo.cpp, built with the library.  It checks the
single-token closed form (decode returns V[0] bit for bit, Section 2.1 with one cached token), the
pool layout the header states, and drains a request stream through the scheduler and the runner
(Section 3.3, Algorithm 3).
"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DEMO = os.path.join(ROOT, "paper_2404_02015_amd", "examples", "c_abi_demo")


def test_demo_is_built():
    assert os.access(DEMO, os.X_OK), "run `python -m paper_2404_02015_amd.build` first"


@pytest.mark.gpu
def test_c_abi_demo_runs_clean():
    print("[case] C ABI demo", flush=True)
    r = subprocess.run([DEMO], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0 and "c_abi_demo OK" in r.stdout
