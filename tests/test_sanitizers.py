"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code (CPU only, no GPU involved):
  * the oracle: oracle.cpp is built with g++ -fsanitize=address,undefined into a library of its own and a slice of
    the oracle's own test-suite runs against it in a child process (the sanitizer runtimes are preloaded there);
  * the library's host core: host.cpp and iter.cpp (validation, type promotion, broadcasting, overlap rules, the operand
    iterator) are built host-only with hipcc and the sanitizers, linked with a driver that sweeps shapes and dtypes.
Any report from either sanitizer fails the test (undefined behaviour is not recoverable in these builds)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_10977_amd", "csrc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
REPORTS = ("ERROR: AddressSanitizer", "runtime error:", "SUMMARY: UndefinedBehaviorSanitizer")


def runtime(name):
    path = subprocess.run(["g++", "-print-file-name=" + name], capture_output=True, text=True, check=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(shutil.which("g++") is None or runtime("libasan.so") is None, reason="g++ with the ASan runtime is needed")
def test_oracle_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "liboracle_san.so")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared"] + SAN +
                   [os.path.join(ROOT, "oracle", "oracle.cpp"), "-o", lib], check=True)
    env = dict(os.environ)
    preload = [runtime("libasan.so"), runtime("libubsan.so")] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env.update(LD_PRELOAD=":".join(p for p in preload if p), ORACLE_LIB=lib, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    check = "from oracle import oracle as O; import sys; sys.exit(0 if O.lib()._name == %r else 3)" % lib
    assert subprocess.run([sys.executable, "-c", check], env=env, cwd=ROOT).returncode == 0, "the sanitized oracle was not the one loaded"
    tests = ["tests/test_oracle_elementwise.py", "tests/test_oracle_reduce.py", "tests/test_oracle_softmax_scan.py",
             "tests/test_oracle_indexing.py", "tests/test_oracle_indexing_more.py", "tests/test_oracle_scatter_reduce_index_put.py",
             "tests/test_oracle_shape_ops.py", "tests/test_oracle_searchsorted.py", "tests/test_oracle_layer_norm_bce.py"]
    p = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider"] + tests, env=env, cwd=ROOT,
                       capture_output=True, text=True)
    out = p.stdout + p.stderr
    assert p.returncode == 0 and not any(r in out for r in REPORTS), out[-4000:]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc is needed")
def test_host_core_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    flags = []
    for f in SAN:
        flags += ["-Xarch_host", f]                  # sanitizers on the host pass only
    cmd = ["hipcc", "-x", "hip", "--cuda-host-only", "-std=c++17", "-O1", "-g"] + flags + \
          ["-I", CSRC, "-I", os.path.join(ROOT, "include"), os.path.join(CSRC, "host.cpp"), os.path.join(CSRC, "iter.cpp"),
           os.path.join(ROOT, "tests", "sanitize_host_driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    p = subprocess.run([exe], env=env, capture_output=True, text=True)
    out = p.stdout + p.stderr
    assert p.returncode == 0 and "host core:" in out and not any(r in out for r in REPORTS), out[-4000:]
