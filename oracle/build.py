"""Compile the C oracle into oracle/libcngp_oracle.so with gcc.

Building the checker is not using it: the product library never links or
loads this file.  -ffp-contract=off keeps the single fp32 multiply of the
coordinate scaling a plain IEEE multiply (no fused multiply-add).
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cngp_oracle.c")
LIB = os.path.join(HERE, "libcngp_oracle.so")


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized() -> str:
    """The oracle with its exerciser (sanitize_main.c) as one program under AddressSanitizer and
    UndefinedBehaviorSanitizer, runtimes linked statically so that nothing has to be preloaded.  Returns the path of
    the program (in the git-ignored _build/ folder at the repository root); tests/test_oracle_pins.py runs it."""
    out_dir = os.path.join(os.path.dirname(HERE), "_build")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "oracle_sanitize_check")
    main = os.path.join(HERE, "sanitize_main.c")
    if os.path.exists(exe) and os.path.getmtime(exe) >= max(os.path.getmtime(SRC), os.path.getmtime(main)):
        return exe
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-o", exe, main, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    import sys
    print(build_sanitized() if "--sanitize" in sys.argv else build(force=True))
