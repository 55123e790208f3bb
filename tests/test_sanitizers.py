"""The CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU):
the C oracle runs its pin tests as a sanitized build, and the library's host logic (greedy
search, register rule, tile order, launch plans, argument checks, the refused-launch path of
every vector-ALU launch plan) runs in a sanitized host build of the C ABI's translation unit."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(cmd, env=None, timeout=600):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=timeout,
                         cwd=ROOT)
    return res.returncode, res.stdout


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    lib = str(tmp_path / "liboracle_san.so")
    rc, out = _run([gcc, "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-o", lib, os.path.join(ROOT, "oracle", "amulet_oracle.c"), "-lm"])
    assert rc == 0, out
    asan = subprocess.check_output([gcc, "-print-file-name=libasan.so"], text=True).strip()
    env = dict(os.environ, LD_PRELOAD=asan, ASAN_OPTIONS="detect_leaks=0", AMULET_ORACLE_LIB=lib,
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    rc, out = _run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_pins.py",
                    "tests/test_oracle_general_pins.py", "tests/test_oracle_f64_pins.py"], env=env)
    assert rc == 0 and " passed" in out and "runtime error" not in out and "AddressSanitizer" not in out, out[-4000:]


def test_host_logic_under_asan_and_ubsan(tmp_path):
    from paper_2305_08872_amd import build as hip_build
    hipcc = hip_build._hipcc()
    if not os.path.exists(os.path.join(hip_build.OBJ_DIR, "amulet_api.o")):
        hip_build.build()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all"]
    api_obj = str(tmp_path / "amulet_api_san.o")
    rc, out = _run([hipcc] + hip_build.HIPCC_FLAGS + san + ["-g", "-c", os.path.join(hip_build.CSRC, "amulet_api.hip"),
                                                            "-o", api_obj])
    assert rc == 0, out[-4000:]
    main_obj = str(tmp_path / "host_logic_main.o")
    rc, out = _run([hipcc] + hip_build.HIPCC_FLAGS + san + ["-g", "-x", "hip", "-c",
                                                            os.path.join(ROOT, "tests", "sanitize", "host_logic_main.cpp"),
                                                            "-o", main_obj])
    assert rc == 0, out[-4000:]
    others = [os.path.join(hip_build.OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in hip_build.SOURCES
              if s != "amulet_api.hip"]
    exe = str(tmp_path / "host_logic_san")
    rc, out = _run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                    "-o", exe, main_obj, api_obj] + others)
    assert rc == 0, out[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    rc, out = _run([exe], env=env)
    assert rc == 0 and "host logic under sanitizers: ok" in out and "runtime error" not in out, out[-4000:]
