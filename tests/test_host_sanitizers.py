"""The C ABI's host code (argument validation, workspace sizing, dispatch) compiled with the address
and undefined-behaviour sanitizers for the host side only and driven through its rejection paths.
Needs the kernels' object files of a previous build (python -c 'import __graft_entry__ as g; g.build()')."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2403_09347_amd")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2403_09347_amd import build as B
    objs = [os.path.join(PKG, "_build", s.replace(".hip", ".o")) for s in B.SOURCES if s != "burst_api.hip"]
    if not all(os.path.exists(o) for o in objs) or not os.path.exists(HIPCC):
        pytest.skip("kernel object files or compilers not available")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    api = str(tmp_path / "api_san.o")
    drv = str(tmp_path / "driver.o")
    exe = str(tmp_path / "driver")
    run = lambda cmd: subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, errors="replace")
    flags = [f for f in B.FLAGS if f != "-O3"]
    run([HIPCC, "-O1", "-g", *flags, *san, "-c", os.path.join(PKG, "csrc", "burst_api.hip"), "-o", api])
    run([HIPCC, "-O1", "-g", *flags, *san, "-I", os.path.join(ROOT, "include"),
         "-c", os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", drv])
    run([HIPCC, "--offload-arch=gfx950", *san, api, drv, *objs, "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, errors="replace", env=env, timeout=120)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "host checks failed: 0" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-3000:]
