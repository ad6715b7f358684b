"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

* The oracle's C source is built with ``-fsanitize=address,undefined`` and every pin of
  ``test_oracle_pins`` / ``test_oracle_next_pins`` is run through that build, in a child process that has
  gcc's sanitizer runtimes loaded first.
* The host side of the HIP library (argument validation, tensor-list layout, launch planning) is
  built with the same sanitizers on the host compilation only and driven by
  ``host_sanitize_driver.cpp``; device code is compiled as usual and never runs.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TESTS = os.path.join(ROOT, "tests")
REPORTS = ("ERROR: AddressSanitizer", "runtime error:", "ERROR: LeakSanitizer")

CHILD = r'''
import sys
sys.path.insert(0, sys.argv[2]); sys.path.insert(0, sys.argv[3])
import oracle
from test_oracle_pins import ALL_CHECKS
from test_oracle_next_pins import NEXT_CHECKS
ora = oracle.Oracle(sys.argv[1])
for check in (*ALL_CHECKS, *NEXT_CHECKS):
    check(ora)
    print("ok", check.__name__, flush=True)
print("pins passed under sanitizers", len(ALL_CHECKS) + len(NEXT_CHECKS))
'''


def gcc_runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    asan, ubsan = gcc_runtime("libasan.so"), gcc_runtime("libubsan.so")
    if not asan or not ubsan:
        pytest.skip("gcc sanitizer runtimes not installed")
    import oracle

    lib = os.path.join(tmp_path, "liboracle_san.so")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-pthread",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-o", lib, oracle.SOURCE]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    # the sanitizer runtimes must come first in the child; anything already preloaded stays behind them
    env["LD_PRELOAD"] = ":".join(p for p in (asan, ubsan, env.get("LD_PRELOAD", "")) if p)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"   # the interpreter itself leaks
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    res = subprocess.run([sys.executable, "-c", CHILD, lib, ROOT, TESTS], capture_output=True, text=True, env=env,
                         timeout=900)
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "pins passed under sanitizers" in res.stdout
    assert not any(r in out for r in REPORTS), out[-4000:]


def test_host_layer_of_the_library_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC") or shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc) and shutil.which(hipcc) is None:
        pytest.skip("hipcc not available")
    exe = os.path.join(tmp_path, "host_sanitize_driver")
    san = []
    for flag in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                 "-fno-omit-frame-pointer"):
        san += ["-Xarch_host", flag]
    cmd = [hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *san, "-o", exe,
           os.path.join(ROOT, "paper_2404_00438_amd", "csrc", "dlion.hip"),
           os.path.join(TESTS, "host_sanitize_driver.cpp")]
    built = subprocess.run(cmd, capture_output=True, text=True, cwd=tmp_path)
    assert built.returncode == 0, built.stderr[-4000:]
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0"         # the HIP runtime keeps its own process-lifetime state
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    try:
        import torch
        if torch.cuda.is_available():
            env["DLION_SANITIZE_EXPECT_GPU"] = "1"   # launches would succeed: skip the calls that rely on a refusal
    except ImportError:
        pass
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "host layer ok" in res.stdout
    assert not any(r in out for r in REPORTS), out[-4000:]
