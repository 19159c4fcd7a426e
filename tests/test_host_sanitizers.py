"""The library's host code (argument checks, workspace carve-up, launch set-up) built with
AddressSanitizer and UndefinedBehaviorSanitizer and walked by a small C driver
(tests/host_checks/abi_driver.c) that calls every entry point of include/sv.h with arguments
the host must reject, and with empty batches.  Device code is compiled as usual (GPU
sanitizers are not available here); nothing is launched, so no GPU is needed."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


@pytest.mark.skipif(shutil.which(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) is None, reason="hipcc not found")
def test_host_code_under_asan_and_ubsan(tmp_path):
    import importlib.util
    spec = importlib.util.spec_from_file_location("_sv_build", os.path.join(ROOT, "paper_2509_24328_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    lib = str(tmp_path / "libsv_san.so")
    flags = [f for f in mod.FLAGS if f != "-O3"] + ["-O1"]
    r = subprocess.run([hipcc] + flags + san + ["-o", lib] + [os.path.join(mod.CSRC, s) for s in mod.SOURCES],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    exe = str(tmp_path / "abi_driver")
    r = subprocess.run([hipcc, "-x", "c", os.path.join(ROOT, "tests", "host_checks", "abi_driver.c"), "-x", "none",
                        "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-g",
                        "-o", exe, lib, f"-Wl,-rpath,{tmp_path}"], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out
    assert "host ABI walk ok" in out and "runtime error" not in out and "AddressSanitizer" not in out, out
