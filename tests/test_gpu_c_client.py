"""The C ABI used from plain C99, with hipMalloc'ed memory and neither Python
nor PyTorch in the process: the client next to the library runs cases with
closed-form results (ASGD for lambda = 0, pull semantics, one delay-compensated
update worked by hand, the synchronous fold in the caller's order and ranked by
norm with the caller's and with the library's static workspace) and the error
paths."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "paper_1609_08326_amd", "abi_client")


def test_plain_c_client_of_the_abi():
    if not os.path.exists(CLIENT):
        raise FileNotFoundError("%s is not built; run `python -m paper_1609_08326_amd.build`" % CLIENT)
    print("running", CLIENT, flush=True)
    sys.stdout.flush()
    p = subprocess.run([CLIENT], capture_output=True, text=True, timeout=100)
    print(p.stdout, p.stderr, flush=True)
    assert p.returncode == 0 and "abi_client: OK" in p.stdout, p.stdout + p.stderr
