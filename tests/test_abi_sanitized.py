"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer.

The host translation unit (csrc/bd_lib.hip: context, planning, weight upload, argument checks, error paths) is compiled
with the sanitizers on its host pass only, linked with the kernel objects of the ordinary build, and driven by the
native program tests/abi_host_check.cpp, which makes the calls of tests/test_abi_cpu.py (a sanitized shared library
cannot be loaded into an unsanitized Python).  No GPU needed; with one present the program also creates and destroys a
context."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2604_06832_amd")
BUILD = os.path.join(PKG, "_build")
SAN = os.path.join(BUILD, "san")
HIPCC = "/opt/rocm/bin/hipcc"
CLANG = "/opt/rocm/lib/llvm/bin/clang++"
KERNEL_UNITS = ["k_stream", "k_mega", "k_prefill", "k_attention"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)), reason="no ROCm compiler here")
def test_host_code_under_asan_and_ubsan():
    if not all(os.path.exists(os.path.join(BUILD, u + ".o")) for u in KERNEL_UNITS):
        import __graft_entry__ as g
        g.build()                                   # leaves the kernel objects in _build/
    os.makedirs(SAN, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Wno-unused-value",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *san,
          "-c", os.path.join(PKG, "csrc", "bd_lib.hip"), "-o", os.path.join(SAN, "bd_lib.o")])
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
          "-fsanitize=undefined", "-shared-libsan", os.path.join(SAN, "bd_lib.o"),
          *[os.path.join(BUILD, u + ".o") for u in KERNEL_UNITS], "-o", os.path.join(SAN, "libbd_san.so")])
    rt_dir = os.path.dirname(_run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"]).strip())
    _run([CLANG, "-std=c++17", "-g", "-O1", "-fsanitize=address", "-fsanitize=undefined",
          "-fno-sanitize-recover=undefined", "-shared-libsan", os.path.join(ROOT, "tests", "abi_host_check.cpp"),
          "-L" + SAN, "-lbd_san", "-Wl,-rpath," + SAN, "-Wl,-rpath," + rt_dir, "-o", os.path.join(SAN, "abi_host_check")])
    # leaks are reported for this library's own allocations; what the ROCm runtime keeps until the process ends is not ours
    supp = os.path.join(SAN, "lsan.supp")
    with open(supp, "w") as f:
        f.write("leak:libhsa-runtime64\nleak:libamdhip64\nleak:libamd_comgr\nleak:libhsakmt\nleak:libdrm\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               LSAN_OPTIONS="suppressions=" + supp + ":print_suppressions=0")
    r = subprocess.run([os.path.join(SAN, "abi_host_check")], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                       env=env, timeout=300)
    assert r.returncode == 0 and "ALL OK" in r.stdout, r.stdout[:1500] + "\n...\n" + r.stdout[-2500:]
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, r.stdout[-4000:]
    shutil.rmtree(SAN, ignore_errors=True)
