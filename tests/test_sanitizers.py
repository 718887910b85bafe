"""Host code under sanitizers, on the CPU.

* The oracle (oracle/hps_oracle.cpp) is built with gcc's AddressSanitizer and
  UndefinedBehaviorSanitizer and the whole oracle test file runs against that build in a child
  process (the sanitizer runtime has to be loaded before the interpreter starts).
* The host side of the HIP library is built with -fsanitize=undefined in trap mode (this
  image ships no clang sanitizer runtime, so undefined behaviour ends the process instead of
  being reported, and there is no AddressSanitizer for it) and the C ABI's argument checks
  (tests/test_abi.py: calls that return before anything touches a GPU) run against that build.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pytest(test_file, env_extra):
    env = dict(os.environ)
    env.update(env_extra)
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", test_file), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True, timeout=600)
    return res.returncode, res.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if not gxx or not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no g++ / libasan here")
    lib = str(tmp_path / "libhps_oracle_san.so")
    subprocess.check_call([gxx, "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", lib,
                           os.path.join(ROOT, "oracle", "hps_oracle.cpp")])
    preload = asan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    rc, out = _run_pytest("test_oracle.py", {"HPS_ORACLE_LIB": lib, "LD_PRELOAD": preload,
                                             "ASAN_OPTIONS": "detect_leaks=0"})
    assert rc == 0 and "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]


def test_abi_argument_checks_with_undefined_behaviour_traps(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    lib = str(tmp_path / "libhps_ubsan.so")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-shared", "-fPIC",
                          "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined",
                          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", lib,
                          os.path.join(ROOT, "paper_2003_05622_amd", "csrc", "hps.hip")],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    rc, out = _run_pytest("test_abi.py", {"HPS_LIB": lib})
    assert rc == 0, out[-4000:]
