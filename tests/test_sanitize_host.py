"""The CPU oracle and the host half of the library, built with -fsanitize=address,undefined
and driven by tests/sanitize/host_driver.cc (random allocator traffic, send ranges, address
runs, prefix index, prep_recv, forks; the oracle's attention and copies).  No GPU involved: the
library's host code is compiled as plain C++, without its kernels."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_and_oracle_under_address_and_ub_sanitizers(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2412_12488_amd", "csrc"),
           "-I", "/opt/rocm/include", "-D__HIP_PLATFORM_AMD__"]
    objs = []
    for name, cmd in (
            ("oracle.o", ["gcc", "-std=c11", "-fopenmp", *san, "-c", os.path.join(ROOT, "oracle", "mc_oracle.c")]),
            ("host.o", ["g++", "-std=c++17", "-x", "c++", *san, *inc, "-c",
                        os.path.join(ROOT, "paper_2412_12488_amd", "csrc", "mc_host.hip")]),
            ("driver.o", ["g++", "-std=c++17", *san, *inc, "-c",
                          os.path.join(ROOT, "tests", "sanitize", "host_driver.cc")])):
        out = str(tmp_path / name)
        subprocess.run(cmd + ["-o", out], check=True, capture_output=True, text=True)
        objs.append(out)
    exe = str(tmp_path / "host_driver")
    subprocess.run(["g++", *san, "-fopenmp", "-o", exe, *objs, "-lm"], check=True,
                   capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "host sanitize run ok" in res.stdout
