"""Compile the HIP sources into paper_2312_17241_amd/libcngp.so for gfx950.

hipcc cross-compiles without a GPU.  Flags: packed fp32 instructions are switched off
(-packed-fp32-ops), floating-point atomics use the hardware instructions
(-munsafe-fp-atomics; all gradient buffers are ordinary coarse-grained device memory).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcngp.so")
SOURCES = ["cngp_api.hip", "cngp_sort.hip"]
HEADERS = ["cngp_device.h", "cngp_kernels.h", "cngp_fwd_level.h", "cngp_bwd_sliced.h", "cngp_bwd_binned.h", "cngp_optim.h", "cngp_mlp.h", "cngp_rates.h", os.path.join("..", "..", "include", "cngp.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, extra=()) -> str:
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra) + ["-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    msgs = [ln for ln in (res.stdout + res.stderr).splitlines()
            if "packed-fp32-ops" not in ln]          # the host pass does not know the feature: harmless
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(msgs))
    if msgs:
        print("\n".join(msgs), file=sys.stderr)
    return LIB


def build_host_sanitized() -> str:
    """The library's host code (validation, plan, workspace layout) with its exerciser csrc/host_check_main.cpp as one
    program, AddressSanitizer and UndefinedBehaviorSanitizer on the HOST side only (the device side is compiled as
    always; nothing of it runs).  About two minutes; the result lives in the git-ignored _build/ folder and is
    rebuilt only when a source is newer.  tests/test_abi.py runs it."""
    out_dir = os.path.join(os.path.dirname(HERE), "_build")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "cngp_host_sanitize_check")
    main = os.path.join(CSRC, "host_check_main.cpp")
    srcs = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [main]
    if os.path.exists(exe) and os.path.getmtime(exe) >= max(os.path.getmtime(f) for f in srcs):
        return exe
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC", "-O3")] + ["-O1", "-g"]
    cmd = [hipcc] + flags + san + ["-o", exe, main] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc (host sanitizers) failed:\n" + "\n".join(
            ln for ln in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in ln))
    return exe


if __name__ == "__main__":
    if "--host-sanitizers" in sys.argv:
        print(build_host_sanitized())
    else:
        print(build(force=True, extra=sys.argv[1:]))
