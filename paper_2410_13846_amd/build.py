"""Builds liblt_hip.so (C-ABI library + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
# LT_HIP_LIBRARY names another build of the same C ABI to load instead (the CPU-only sanitizer build of the host layer
# that the test-suite makes); it is never built or rebuilt from here.
LIB_PATH = os.environ.get("LT_HIP_LIBRARY") or os.path.join(_HERE, "liblt_hip.so")
SOURCES = ["lt_api.cpp", "lt_decode.hip", "lt_score.hip", "lt_prefill.hip"]
HEADERS = ["lt_kernels.h", os.path.join("..", "..", "include", "lt.h"), os.path.join("..", "..", "include", "lt_measure.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # an atomic issued by one lane stays one instruction whose result is waited for where it is used (the
    # wave-level rewrite of atomics reads the result back on the spot, which stalls a software pipeline)
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > built for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library (always when force=True; otherwise only if missing).  The translation units are
    compiled side by side, then linked."""
    if os.environ.get("LT_HIP_LIBRARY"):
        return LIB_PATH                         # somebody else's build: used as it is (loading fails if it is absent)
    if not force and os.path.exists(LIB_PATH):
        return LIB_PATH
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    messages = []

    def run(cmd):
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        lines = [l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l]
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
        messages.extend(lines)

    with tempfile.TemporaryDirectory(prefix="lt_build_") as tmpdir:
        objects = [os.path.join(tmpdir, os.path.splitext(f)[0] + ".o") for f in SOURCES]
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            list(pool.map(lambda so: run([hipcc] + compile_flags + ["-c", os.path.join(CSRC, so[0]), "-o", so[1]]),
                          zip(SOURCES, objects)))
        tmp = LIB_PATH + ".tmp.%d" % os.getpid()
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objects + ["-o", tmp])
    if verbose and messages:
        print("\n".join(messages))
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build(force=True, verbose=True))
