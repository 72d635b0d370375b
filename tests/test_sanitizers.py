"""CPU sanitizer pass over everything of this repository that runs on the host: the library's host layer
(csrc/lt_api.cpp, built against stub launchers instead of the kernels) and the oracle (oracle/lt_oracle.c), both
compiled with -fsanitize=address,undefined, and exercised by the host-API, host-logic and oracle tests in a child
process that loads those builds.  GPU code is not covered (sanitizers for device code are not available here)."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-fPIC", "-shared"]


@pytest.fixture(scope="module")
def sanitized_libraries(tmp_path_factory):
    out = tmp_path_factory.mktemp("san")
    host = str(out / "liblt_host_san.so")
    orc = str(out / "liblt_oracle_san.so")
    csrc = os.path.join(ROOT, "paper_2410_13846_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN +
                   ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + csrc,
                    os.path.join(csrc, "lt_api.cpp"), os.path.join(ROOT, "tests", "stubs", "lt_stub_launchers.cpp"), "-o", host],
                   check=True, timeout=600)
    subprocess.run(["gcc", "-Wall", "-Wextra", "-fopenmp"] + SAN + [os.path.join(ROOT, "oracle", "lt_oracle.c"), "-o", orc, "-lm"],
                   check=True, timeout=600)
    return host, orc


def test_host_layer_and_oracle_under_address_and_undefined_behaviour_sanitizers(sanitized_libraries):
    host, orc = sanitized_libraries
    asan_rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    env = dict(os.environ)
    # the sanitizer runtime has to be the first library of the (uninstrumented) interpreter; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join(x for x in (asan_rt, env.get("LD_PRELOAD", "")) if x)
    # the interpreter itself is not leak-clean; leaks of the two libraries are looked for by the tests that destroy what they create
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["LT_HIP_LIBRARY"] = host
    env["LT_ORACLE_LIBRARY"] = orc
    env["OMP_NUM_THREADS"] = env.get("OMP_NUM_THREADS", "4")
    tests = ["tests/test_host_api.py", "tests/test_host_logic.py", "tests/test_oracle_decode.py", "tests/test_oracle_ratio.py",
             "tests/test_oracle_select.py", "tests/test_oracle_prefill.py"]
    run = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-rA", "-m", "not gpu", "-p", "no:cacheprovider"] + tests,
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    report = run.stdout + run.stderr
    assert run.returncode == 0, report[-6000:]
    assert "ERROR: AddressSanitizer" not in report and "runtime error:" not in report, report[-6000:]
    # the child really ran against the stub build: the host-logic tests are skipped anywhere else
    passed = re.findall(r"^PASSED tests/test_host_logic\.py::", report, flags=re.M)
    assert len(passed) >= 12, report[-3000:]
    assert not re.search(r"^SKIPPED .*test_host_logic", report, flags=re.M), report[-3000:]
