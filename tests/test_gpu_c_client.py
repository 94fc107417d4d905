"""The C ABI used from plain C (tests/c_client/verify_step.c, built by __graft_entry__.build()):
attention against closed forms, greedy acceptance and compaction, with no Python or PyTorch in the
process that calls the library."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
BIN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_client", "verify_step")


def test_plain_c_client_runs_a_verification_step():
    assert os.path.exists(BIN), "build the C client first: python -c 'import __graft_entry__ as g; g.build()'"
    r = subprocess.run([BIN], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert r.stdout.strip().endswith("c client ok")
