"""The library driven from a plain C host program with hipMalloc'd buffers and no Python in the process
(tests/host_c/des_host_step.c, built by __graft_entry__.build()): find with insert, forward partials, the
three aggregations, FM finalize, merged Adagrad update and key export, each checked inside the program against
the C oracle linked into it.  This test only runs the program and relays its verdict."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BIN = os.path.join(ROOT, "tests", "host_c", "des_host_step")


def test_plain_c_host_program_matches_oracle():
    if not os.path.exists(BIN):
        pytest.fail("tests/host_c/des_host_step is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    print("running the plain C host program", flush=True)
    res = subprocess.run([BIN], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=110)
    print(res.stdout, flush=True)
    assert res.returncode == 0, res.stdout[-2000:]
    assert "des_host_step: PASS" in res.stdout and "FAIL" not in res.stdout
