"""The C ABI's host code (argument validation, workspace planning) under AddressSanitizer and
UndefinedBehaviorSanitizer: api.hip is compiled with both on the host side, linked with a small
driver and the built library's kernel launchers, and run.  CPU only; nothing reaches the GPU."""
import os
import shutil
import subprocess

import pytest

from paper_2602_05885_amd import binding as B
from paper_2602_05885_amd import build as pgbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(not os.path.exists(CLANG) or shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs the ROCm compilers")
def test_argument_layer_is_clean_under_asan_and_ubsan(tmp_path):
    assert os.path.exists(B.LIB_PATH), "build the library first"
    api_o, drv_o, exe = (str(tmp_path / n) for n in ("api_san.o", "driver.o", "abi_san"))
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]
    flags = [f for f in pgbuild.FLAGS if f != "-O3"]
    run = lambda cmd: subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    run([pgbuild.hipcc(), "-O1", "-g", *flags, f"-I{ROOT}/include", *host_san, "-c",
         os.path.join(pgbuild.CSRC, "api.hip"), "-o", api_o])
    sym = subprocess.run(["nm", api_o], stdout=subprocess.PIPE, text=True).stdout
    assert "__asan" in sym and "__ubsan" in sym, "host code was not instrumented"
    run([CLANG, "-O1", "-g", "-std=c++17", f"-I{ROOT}/include", *SAN, "-c",
         os.path.join(ROOT, "tests", "abi_sanitize_driver.cpp"), "-o", drv_o])
    pkg = os.path.dirname(B.LIB_PATH)
    run([CLANG, "-fsanitize=address", "-fsanitize=undefined", api_o, drv_o, f"-L{pkg}", "-l:libpg_head.so",
         "-L/opt/rocm/lib", "-lamdhip64", f"-Wl,-rpath,{pkg}", "-Wl,-rpath,/opt/rocm/lib", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120, env=env)
    assert r.returncode == 0 and "(0 failures)" in r.stdout, r.stdout[-2000:]
