"""Host code of the C ABI (iso_api.hip, iso_bind.hpp: handles, device tables, graphs, the static
scratch array) without a GPU: compiled for the host only, linked against a stand-in HIP runtime
(tests/hip_stub_runtime.cpp) and driven through the life cycle of every kind of request under
AddressSanitizer and LeakSanitizer.  The same build with a leak planted in iso_request_free (its
hipFree renamed to a function that frees nothing) must fail."""
import os
import subprocess
import tempfile

import pytest

from conftest import ROOT

CSRC = os.path.join(ROOT, "paper_1606_07676_amd", "csrc")
CLANGXX = "/opt/rocm/llvm/bin/clang++"


def _build(td, tag, extra):
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    common = ["-O1", "-g", "-std=c++17", "-fsanitize=address", "-fno-omit-frame-pointer"]
    objs = []
    for src, hip in ((os.path.join(CSRC, "iso_api.hip"), True), (os.path.join(ROOT, "tests", "hip_stub_runtime.cpp"), False),
                     (os.path.join(CSRC, "iso_plan.cpp"), False),
                     (os.path.join(ROOT, "tests", "request_lifecycle_driver.cpp"), False)):
        obj = os.path.join(td, f"{tag}_{os.path.basename(src)}.o")
        if hip:      # the host pass of the HIP compiler: kernels become launch stubs, no device code
            cmd = ["hipcc", "--cuda-host-only", "-fuse-cuid=none", *common, *inc, *extra, "-c", src, "-o", obj]
        else:
            cmd = [CLANGXX, *common, *inc, "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-c", src, "-o", obj]
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert proc.returncode == 0, proc.stdout[-3000:]
        objs.append(obj)
    exe = os.path.join(td, f"lifecycle_{tag}")
    proc = subprocess.run([CLANGXX, "-fsanitize=address", *objs, "-o", exe], stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout[-3000:]
    return exe


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    return subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)


@pytest.mark.skipif(not os.path.exists(CLANGXX), reason="needs the ROCm clang++")
def test_request_life_cycle_leaves_nothing_behind_and_a_planted_leak_is_caught():
    with tempfile.TemporaryDirectory() as td:
        good = _run(_build(td, "good", []))
        assert good.returncode == 0, good.stdout[-3000:]
        assert "lifecycle ok" in good.stdout and "LeakSanitizer" not in good.stdout
        assert int(good.stdout.split("lifecycle ok:")[1].split()[0]) >= 40
        # iso_request_free (and every other release of a device table) calls a hipFree that frees nothing
        bad = _run(_build(td, "planted", ["-DhipFree=stub_forgetful_free"]))
        assert bad.returncode != 0
        assert "left behind" in bad.stdout and "device allocations" in bad.stdout
        assert "LeakSanitizer: detected memory leaks" in bad.stdout
