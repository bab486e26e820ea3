"""The library's host code (page lists, budgets, policies, buddy allocator, staging ring, allocation solver) under
AddressSanitizer and UndefinedBehaviorSanitizer: tests/host_fuzz.cpp drives accounting-only caches through some
hundred thousand random calls, valid and invalid.  Host code only; nothing here touches a GPU."""
import os
import shutil
import subprocess

import pytest

import paper_2505_18610_amd as kq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_18610_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    inc = os.path.join(ROOT, "include")
    libdir = os.path.dirname(kq.library_path())
    host_o, fuzz_o, exe = tmp_path / "kvq_host.san.o", tmp_path / "host_fuzz.o", tmp_path / "host_fuzz"
    arch_host = [a for f in SAN for a in ("-Xarch_host", f)]
    base = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-I", inc]
    steps = [
        # the library's host translation unit, instrumented on the host side only
        base + ["-x", "hip", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *arch_host,
                "-c", os.path.join(CSRC, "kvq_host.cpp"), "-o", str(host_o)],
        base + ["-x", "hip", *arch_host, "-c", os.path.join(ROOT, "tests", "host_fuzz.cpp"), "-o", str(fuzz_o)],
        # the kernels' launchers (never called without an arena) come from the built library
        [HIPCC, "--offload-arch=gfx950", *SAN, str(fuzz_o), str(host_o), "-o", str(exe), "-L", libdir, "-lkvq",
         "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"],
    ]
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
        if r.returncode != 0 and "sanitize" in r.stderr and "unsupported" in r.stderr:
            pytest.skip("this toolchain has no host sanitizers: " + r.stderr[-200:])
        assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe), "300"], capture_output=True, text=True, timeout=600, env=env)
    if r.returncode != 0 and "ASan runtime does not come first" in r.stderr:
        pytest.skip("a preloaded library keeps the sanitizer runtime from starting")
    assert r.returncode == 0, (r.returncode, r.stdout[-500:], r.stderr[-3000:])
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
    assert r.stdout.startswith("ops "), r.stdout
