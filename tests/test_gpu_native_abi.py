"""The C ABI without Python in the way: tests/native/abi_gpu_check is a plain HIP host program (system HIP
runtime, no framework) that materialises, attaches, swaps and detaches through libtidal and compares every
state bit for bit with the oracle library it links as its checker.  Built by __graft_entry__.build()
(python -m tests.native.build_native); this test only runs it."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "abi_gpu_check")


def test_c_program_drives_the_abi_and_matches_the_oracle():
    assert os.path.exists(EXE), "%s is missing: run `python -m tests.native.build_native` (or __graft_entry__.build())" % EXE
    p = subprocess.run([EXE], capture_output=True, text=True, timeout=100)
    print(p.stdout, flush=True)
    assert p.returncode == 0, (p.returncode, p.stdout[-2000:], p.stderr[-2000:])
    for step in ("materialize", "attach", "swap", "detach", "after rejected calls"):
        assert "%s: bit-exact" % step in p.stdout
    assert "abi gpu check ok" in p.stdout
