"""The host side of libgrpo (argument validation, workspace layout, kernel-plan and chunk logic:
everything tests/test_abi_cpu.py drives) under AddressSanitizer and UndefinedBehaviorSanitizer.

The library's translation unit is compiled for the host only (seconds instead of the minutes the
94 device kernels take) with -fsanitize=address,undefined on the host pass, linked against an
empty stand-in for the device image, and test_abi_cpu.py is run against that build in a child
process with the sanitizer runtime preloaded.  Nothing here launches a kernel, on any machine:
those tests stop at validation.  Any out-of-bounds access, overflow or invalid enum load in the
host code aborts the child.
"""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2505_07291_amd", "csrc", "grpo.hip")


def test_abi_tests_pass_on_a_host_build_with_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    runtimes = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not os.path.exists(hipcc) or not runtimes:
        pytest.skip("hipcc or its sanitizer runtime is not installed here")
    tmp = str(tmp_path)
    obj, stub_c, stub_o, lib = (os.path.join(tmp, f) for f in ("grpo_host.o", "stub.c", "stub.o", "libgrpo_san.so"))
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    cc = subprocess.run([hipcc, "--offload-arch=gfx950", "--offload-host-only", "-O1", "-g", "-std=c++17", "-fPIC",
                         "-c"] + san + ["-I", os.path.join(ROOT, "include"), "-o", obj, SRC],
                        capture_output=True, text=True)
    assert cc.returncode == 0, cc.stderr[-3000:]
    # the host object refers to the device image by one symbol; an empty image stands in for it
    syms = subprocess.run(["nm", obj], capture_output=True, text=True).stdout
    fatbin = [l.split()[-1] for l in syms.splitlines() if " U __hip_fatbin" in l]
    assert len(fatbin) == 1 and "__asan_" in syms and "__ubsan_" in syms, "not the instrumented host object expected"
    with open(stub_c, "w") as f:
        f.write('__attribute__((aligned(4096))) const char %s[4096] = "__CLANG_OFFLOAD_BUNDLE__";\n' % fatbin[0])
    assert subprocess.run(["gcc", "-fPIC", "-c", stub_c, "-o", stub_o]).returncode == 0
    ld = subprocess.run([hipcc, "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                         "-o", lib, obj, stub_o], capture_output=True, text=True)
    assert ld.returncode == 0, ld.stderr[-3000:]

    preload = ":".join(p for p in (runtimes[0], os.environ.get("LD_PRELOAD", "")) if p)
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1", LD_PRELOAD=preload,
               ASAN_OPTIONS="detect_leaks=0:alloc_dealloc_mismatch=0:verify_asan_link_order=0:halt_on_error=1:exitcode=97",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1:exitcode=98")
    child = ("import sys\n"
             "import paper_2505_07291_amd.build as b\n"
             "b.LIB_PATH = %r\n"
             "import pytest\n"
             "sys.exit(pytest.main(['-x', '-q', '-s', '-p', 'no:cacheprovider', 'tests/test_abi_cpu.py']))\n" % lib)
    run = subprocess.run([sys.executable, "-c", child], cwd=ROOT, env=env, capture_output=True, text=True)
    out = run.stdout[-4000:] + run.stderr[-4000:]
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out
    assert run.returncode == 0 and " passed" in run.stdout, out
