"""The library's host logic under AddressSanitizer and UndefinedBehaviorSanitizer.

Builds the library a second time with the sanitizers on its HOST code (device code as usual), builds
tests/host_sanitizer_driver.cpp against it, and runs the driver in a child process: subset rank / unrank over
every index, workspace planning over a grid of shapes, and the argument-error path of every entry point.  The
driver launches no kernel; a sanitizer report or a failed check makes it exit non-zero.  No GPU needed."""
import os
import subprocess

from paper_2402_14800_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = os.path.join(os.path.dirname(os.path.realpath(build.HIPCC)), "..", "lib", "llvm", "bin", "clang++")


def test_host_logic_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = build.build(sanitize=True)
    libdir = os.path.dirname(lib)
    exe = str(tmp_path / "host_sanitizer_driver")
    clang = CLANG if os.path.exists(CLANG) else "/opt/rocm/lib/llvm/bin/clang++"
    cmd = [clang, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-shared-libsan", "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
           "-o", exe, "-L", libdir, "-lmoeprune_hostsan", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib",
           "-Wl,-rpath," + os.path.dirname(subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"],
                                                          capture_output=True, text=True).stdout.strip())]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout[-4000:], r.stderr[-4000:])
    assert "all checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
