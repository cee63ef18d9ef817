"""The C ABI called from a C++ driver whose copy of the library's host code is built
with AddressSanitizer and UndefinedBehaviorSanitizer (tests/abi_sanitizer_driver.cpp):
several hundred small collectives, all algorithms, regular, irregular and mesh, with
the error paths, each result compared with the plain definition inside the driver."""
import os
import subprocess

import pytest

from conftest import ROOT

pytestmark = pytest.mark.gpu

DRIVER = os.path.join(ROOT, "tests", "abi_sanitizer_driver")


def test_c_abi_host_code_is_clean_under_asan_and_ubsan():
    if not os.path.exists(DRIVER):
        pytest.skip("tests/abi_sanitizer_driver is not built (run __graft_entry__.build())")
    env = dict(os.environ)
    # leak checking would report the HIP runtime's own process-lifetime allocations
    env["ASAN_OPTIONS"] = "detect_leaks=0:protect_shadow_gap=0:verify_asan_link_order=0"
    out = subprocess.run([DRIVER], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         timeout=100)
    assert out.returncode == 0, out.stdout[-3000:]
    assert "all ok" in out.stdout
    assert int(out.stdout.rsplit("all ok:", 1)[1].split()[0]) > 500
