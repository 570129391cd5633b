"""The C ABI from plain C: tests/c_client/ccd_client.c (gcc, C99, no Python or torch in the process) fills a pot, calls
ccd_compress and checks return codes, ascending indices, kept NuC slots and bit-exact rows by itself."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

CLIENT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2410_01518_amd", "ccd_client")


def test_plain_c_client_compresses_a_pot():
    if not os.path.exists(CLIENT):
        pytest.skip("the C client is not built: python -m paper_2410_01518_amd.build")
    r = subprocess.run([CLIENT], capture_output=True, text=True, timeout=100)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0 and "ccd_client ok" in r.stdout
