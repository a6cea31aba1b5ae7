"""The plain-C example (paper_2603_28458_amd/csrc/example_decode.c) runs a decode step through the C
ABI with no Python in between and checks the invariants of its own result; here it is run as a
child process and must report success."""
import os
import subprocess

import pytest

from paper_2603_28458_amd import build as B

pytestmark = pytest.mark.gpu


def test_plain_c_example_runs_and_passes_its_own_checks(tmp_path):
    exe = B.EXAMPLE_PATH
    if not os.path.exists(exe):
        exe = B.build_example(verbose=False, out_path=str(tmp_path / "example_decode"))
    print(f"\n[c-example] {exe}", flush=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(res.stdout, flush=True)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "example ok" in res.stdout
