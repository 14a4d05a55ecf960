"""The host logic of the C-ABI library (tova_api.cpp: validation, layout, launch planning, launch loops)
built for the CPU with AddressSanitizer and UndefinedBehaviorSanitizer against stand-ins for the device
side (tests/host_sanitizer/stubs.cpp) and driven through the C ABI by tests/host_sanitizer/driver.cpp.
No GPU, no HIP runtime: sanitizers run on host code only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_06104_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitizer")


def test_host_logic_under_asan_and_ubsan(tmp_path):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "host_sanitizer")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "tova_api.cpp"), os.path.join(HERE, "stubs.cpp"), os.path.join(HERE, "driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    for v in [x for x in env if x.startswith("TOVA_")]:
        env.pop(v)
    # (whatever the environment preloads stays; ASan is told not to insist on being first in the list)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all as expected" in r.stdout
