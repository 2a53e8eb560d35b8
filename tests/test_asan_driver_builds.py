"""The host-side memory-checking driver (tests/asan_driver.cpp) walks through every entry point
of the C ABI; it is run by hand on a GPU machine under AddressSanitizer.  Here it is at least
compiled (host pass only, against the header) so that it cannot fall behind the ABI."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not (os.path.exists(HIPCC) or shutil.which("hipcc")), reason="no hipcc here")
def test_asan_driver_compiles_against_the_header(tmp_path):
    out = tmp_path / "asan_driver.o"
    cmd = [HIPCC if os.path.exists(HIPCC) else "hipcc", "--offload-arch=gfx950", "-std=c++17", "-O0",
           "-Wall", "-Werror", "-I" + os.path.join(ROOT, "include"), "-c",
           os.path.join(ROOT, "tests", "asan_driver.cpp"), "-o", str(out)]
    subprocess.check_call(cmd)
    assert out.exists()
    # every entry point the header declares is exercised by the driver (the measurement aid and
    # the error-message getter included); the allocation-free clustering call needs device
    # arrays and has a GPU test of its own
    import re
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "alpa_dp.h")).read(), flags=re.S)
    declared = set(re.findall(r"\b(alpa_(?:dp|cluster|place)_[a-z_A-Z]+)\s*\(", text))
    src = open(os.path.join(ROOT, "tests", "asan_driver.cpp")).read()
    missing = {n for n in declared if n + "(" not in src} - {"alpa_cluster_layers_static",
                                                             "alpa_dp_solve_dev", "alpa_dp_set_stream"}
    assert not missing, missing
