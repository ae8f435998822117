"""The library's host-only code (layout reformatting, permutation, transpose) and the C oracle under
AddressSanitizer + UndefinedBehaviorSanitizer: a small C++ driver is built with g++ -fsanitize=address,undefined
and run on random inputs; any sanitizer report or broken invariant fails the test.  No GPU code is involved."""
import os
import shutil
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    gxx, gcc = shutil.which("g++"), shutil.which("gcc")
    assert gxx and gcc, "g++ / gcc are part of the image"
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_o = tmp_path / "oracle.o"
    r = subprocess.run([gcc, *san, "-fopenmp", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "spmm_oracle.c"), "-o",
                        str(oracle_o)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    exe = tmp_path / "driver"
    csrc = os.path.join(ROOT, "paper_2412_08902_amd", "csrc")
    # loa.cpp includes the library's internal header, which needs the HIP runtime's types only by name
    r = subprocess.run([gxx, *san, "-std=c++17", "-fopenmp", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), "-I", csrc,
                        "-I", "/opt/rocm/include", os.path.join(csrc, "loa.cpp"),
                        os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"), str(oracle_o), "-o", str(exe)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ)
    # a preloaded library may come before the sanitizer runtime in the link order; that is fine here.  Leak checking
    # needs ptrace, which containers often deny.
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "host sanitize driver: ok" in r.stdout
