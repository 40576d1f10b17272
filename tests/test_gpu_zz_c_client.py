"""The C ABI used from plain C (no Python, no torch in the process): tests/c_client/acc_client.c."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_client", "acc_client")


def test_plain_c_client_runs_the_layer():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    assert os.path.exists(EXE), "tests/c_client/acc_client is not built: run __graft_entry__.build()"
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, (r.stdout, r.stderr)
    assert "C client OK" in r.stdout
