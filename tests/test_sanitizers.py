"""CPU sanitizer pass: the oracle (plain C) and the library's host-only code
(generators, validation, walk builders of csrc/host_perm.hip) are rebuilt for
the CPU with AddressSanitizer and UndefinedBehaviorSanitizer, and the existing
pins are run against those builds in processes of their own.  Nothing here
touches a GPU."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1611_04581_amd", "csrc")


def _asan_runtime():
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no gcc")
    path = subprocess.run([gcc, "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    return os.path.realpath(path)


def _env(**extra):
    env = dict(os.environ)
    env["LD_PRELOAD"] = _asan_runtime()
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    env.update(extra)
    return env


def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    from oracle import build as obuild
    lib = obuild.build_sanitized(str(tmp_path / "liboracle_san.so"))
    files = ["tests/test_oracle_steps.py", "tests/test_oracle_variants.py", "tests/test_oracle_async.py",
             "tests/test_oracle_special.py", "tests/test_oracle_rng.py"]
    done = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files], cwd=ROOT,
                          env=_env(GSGD_ORACLE_LIB=lib), capture_output=True, text=True, timeout=900)
    assert done.returncode == 0, done.stdout[-3000:] + done.stderr[-3000:]
    assert "ERROR: AddressSanitizer" not in done.stderr and "runtime error" not in done.stderr


def test_host_generators_and_walk_builders_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if not gxx:
        pytest.skip("no g++")
    rocm_inc = "/opt/rocm/include"
    lib = str(tmp_path / "libhostperm_san.so")
    # host_perm.hip holds no device code: it compiles as plain C++ against the HIP headers
    subprocess.run([gxx, "-x", "c++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared", "-fPIC",
                    "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", rocm_inc,
                    os.path.join(CSRC, "host_perm.hip"), "-o", lib], check=True)
    done = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "san_host_driver.py"), lib], cwd=ROOT,
                          env=_env(), capture_output=True, text=True, timeout=900)
    assert done.returncode == 0, done.stdout[-3000:] + done.stderr[-3000:]
    assert "clean under the sanitizers" in done.stdout
    assert "ERROR: AddressSanitizer" not in done.stderr and "runtime error" not in done.stderr
