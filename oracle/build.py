"""Compile the CPU oracle (plain C) into oracle/libdlcx_oracle.so.

Test infrastructure: the oracle is only ever loaded by tests/, the smoke check
and the bench's cpu_baseline leg.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dlcx_oracle.c")
OUT = os.path.join(HERE, "libdlcx_oracle.so")
CHECK_SRC = os.path.join(HERE, "sanitize_check.c")
CHECK_OUT = os.path.join(HERE, "sanitize_check")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", OUT, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


def build_sanitized() -> str:
    """The oracle and its driver sanitize_check.c as one program under AddressSanitizer and
    UndefinedBehaviorSanitizer (host code only).  Running it exercises every oracle function on
    exact-size heap blocks; any report ends it with a non-zero status."""
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
           "-o", CHECK_OUT, CHECK_SRC, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return CHECK_OUT


if __name__ == "__main__":
    print(build(force=True))
    if "--sanitize" in sys.argv:
        exe = build_sanitized()
        sys.exit(subprocess.run([exe]).returncode)
    sys.exit(0)
