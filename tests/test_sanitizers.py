"""AddressSanitizer + UndefinedBehaviorSanitizer over the CPU side: the oracle's C source and the host side of
the library (validation, planning, work split, C ABI; device launchers replaced by stand-ins) are built with
gcc's sanitizers and the host-only test files run against those builds in a child process.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2506_17255_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
SUITE = ["tests/test_oracle_pins.py", "tests/test_oracle_lowbit.py", "tests/test_library_host.py", "tests/test_prefill_split.py",
         "tests/test_layer_file.py", "tests/test_decode_plan.py"]


def _runtime():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _preload_in_use():
    if os.environ.get("LD_PRELOAD"):
        return True
    try:
        return bool(open("/etc/ld.so.preload").read().strip())
    except OSError:
        return False


@pytest.mark.skipif(os.environ.get("SKETCH_ORACLE_LIB") is not None, reason="already inside the sanitizer run")
def test_cpu_suite_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan = _runtime()
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    if _preload_in_use():
        pytest.skip("another preloaded library is in use; the sanitizer runtime has to come first")
    oracle_so = tmp_path / "liboracle_san.so"
    subprocess.check_call(["gcc", "-std=c11", "-fPIC", "-shared", *SAN, "-o", str(oracle_so),
                           os.path.join(ROOT, "oracle", "sketch_oracle.c"), "-lm"])
    host_so = tmp_path / "libsketch_linear_host_san.so"
    subprocess.check_call(["g++", "-std=c++17", "-fPIC", "-shared", *SAN, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", str(host_so),
                           os.path.join(CSRC, "skl_host.cpp"), os.path.join(CSRC, "skl_file.cpp"),
                           os.path.join(ROOT, "tests", "sanitize", "host_stubs.cpp"),
                           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    env = dict(os.environ, LD_PRELOAD=asan, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1", SKETCH_ORACLE_LIB=str(oracle_so), SKETCH_LINEAR_LIB=str(host_so))
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *SUITE], cwd=ROOT, env=env,
                         capture_output=True, text=True, timeout=1500)
    report = res.stdout[-4000:] + res.stderr[-4000:]
    assert res.returncode == 0, report
    assert "AddressSanitizer" not in report and "runtime error" not in report, report
    assert " passed" in res.stdout
