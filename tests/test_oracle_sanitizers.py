"""The fp64 CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

A private copy of oracle/ is compiled with gcc's -fsanitize=address,undefined and the four
pin files are run against that copy in a child process (the sanitizer runtime has to be the
first library the interpreter loads, hence the child and its LD_PRELOAD).  Any out-of-bounds
access, use after free, signed overflow, misaligned or null access, or invalid shift in the
oracle's C code aborts the child.  Host code only: nothing here touches the GPU library.
"""
import os
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["test_oracle_pins.py", "test_oracle_aux_pins.py", "test_oracle_rewards_pins.py",
        "test_oracle_lmhead_pins.py"]
SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
             "-g", "-O1"]


def _runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    asan = _runtime("libasan.so")
    assert asan, "gcc's libasan.so not found: this image's gcc is expected to ship it"
    tmp = str(tmp_path)
    os.makedirs(os.path.join(tmp, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(tmp, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "*.tmp.*", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(tmp, "tests", "golden"))
    for f in ["conftest.py"] + PINS:
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(tmp, "tests", f))
    src = os.path.join(tmp, "oracle", "grpo_oracle.c")
    lib = os.path.join(tmp, "oracle", "libgrpo_oracle.so")
    cc = subprocess.run(["gcc", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"] + SAN_FLAGS +
                        ["-o", lib, src, "-lm"], capture_output=True, text=True)
    assert cc.returncode == 0, cc.stderr
    # the library really is instrumented (otherwise a clean run would prove nothing)
    syms = subprocess.run(["nm", "-D", "--undefined-only", lib], capture_output=True, text=True).stdout
    assert "__asan_report_load" in syms and "__ubsan_handle" in syms

    preload = ":".join(p for p in (asan, os.environ.get("LD_PRELOAD", "")) if p)
    env = dict(os.environ, PYTHONPATH=tmp, OMP_NUM_THREADS="2", PYTHONDONTWRITEBYTECODE="1", LD_PRELOAD=preload,
               # the interpreter and numpy/torch are not instrumented: leak reports and allocator
               # pairing checks would be about them, not about the oracle
               ASAN_OPTIONS="detect_leaks=0:alloc_dealloc_mismatch=0:verify_asan_link_order=0:"
                            "halt_on_error=1:abort_on_error=0:exitcode=97",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1:exitcode=98")
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] +
                         [os.path.join("tests", f) for f in PINS], cwd=tmp, env=env, capture_output=True, text=True)
    out = run.stdout[-3000:] + run.stderr[-3000:]
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out
    assert run.returncode == 0 and " passed" in run.stdout, out
