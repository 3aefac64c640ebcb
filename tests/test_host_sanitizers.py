"""The host-only code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

oracle/oracle.c and csrc/prefix_tree.cpp do manual index arithmetic (and the tree holds references
into growing vectors); tests/host_sanitize/driver.cpp runs the oracle's entry points on a small paged
workload (bf16 and fp8, including the fp8 append's re-encode branch) and a random session on the
prefix tree, all compiled with -fsanitize=address,undefined.  Any report fails the run.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="needs gcc and g++")
def test_oracle_and_prefix_tree_are_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    obj = str(tmp_path / "oracle.o")
    exe = str(tmp_path / "driver")
    subprocess.run(["gcc", "-std=c11", "-fopenmp", *san, "-c", os.path.join(ROOT, "oracle", "oracle.c"), "-o", obj],
                   check=True, capture_output=True, text=True)
    subprocess.run(["g++", "-std=c++17", "-fopenmp", *san, os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"),
                    os.path.join(ROOT, "paper_2508_11553_amd", "csrc", "prefix_tree.cpp"), obj, "-o", exe, "-lm"],
                   check=True, capture_output=True, text=True)
    env = dict(os.environ, OMP_NUM_THREADS="4",
               # another preloaded library may precede the ASan runtime in the link order; that is harmless here
               ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitizer driver: OK" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
