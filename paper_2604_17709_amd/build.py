"""Build step of the HIP library: one hipcc invocation, gfx950 only, in-tree output.

    python -m paper_2604_17709_amd.build          # compile libdeinfer.so next to this file

The shared object is built in-tree so that it travels with the source snapshot to the
GPU machine; nothing is compiled at import time.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdeinfer.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-munsafe-fp-atomics",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def sources():
    return [os.path.join(CSRC, "deinfer_api.hip")]


SAN_LIB = os.path.join(HERE, "libdeinfer_hostsan.so")
# sanitizers on the host pass only (validation, planning, the host scan of the paged cache): each
# -fsanitize= option directly after -Xarch_host; the device code is compiled as usual
HOST_SANITIZE_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                       "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def asan_runtime() -> str:
    """clang's AddressSanitizer runtime, to preload into a process that loads the host-sanitized build."""
    out = subprocess.run([hipcc(), "--print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(out) or not os.path.exists(out):
        import glob
        cands = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        if not cands:
            raise RuntimeError("clang's asan runtime not found")
        out = cands[0]
    return out


def build_host_sanitized(verbose: bool = False) -> str:
    """libdeinfer_hostsan.so: the same sources with ASan + UBSan on the host code (rebuilt when a source is newer)."""
    srcs = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(os.path.dirname(HERE), "include", "deinfer.h")]
    if os.path.exists(SAN_LIB) and all(os.path.getmtime(SAN_LIB) >= os.path.getmtime(f) for f in srcs):
        return SAN_LIB
    return build_library(verbose=verbose, extra_flags=HOST_SANITIZE_FLAGS, out=SAN_LIB, check_load=False)


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB, check_load: bool = True) -> str:
    LIB = out
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(os.path.dirname(HERE), "include"),
           "-o", LIB + ".tmp", *sources()]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    # a missing host stub or symbol shows up only at load time: check before replacing the old build
    if check_load:
        import ctypes
        try:
            ctypes.CDLL(LIB + ".tmp")
        except OSError as e:
            raise RuntimeError("built library does not load: %s" % e)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
