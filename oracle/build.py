"""Compile the CPU oracle (plain C) into oracle/libqes_oracle.so.

Test infrastructure: building the checker is not using it. The flags are part of the oracle's
definition: -ffp-contract=off keeps gcc from fusing a*b+c on its own, so the only fused
operations are the fmaf() calls written in the source.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "qes_oracle.c")
LIB = os.path.join(HERE, "libqes_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-Wall", "-Wextra",
           "-shared", "-fPIC", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_driver(out_dir: str, sanitized: bool) -> str:
    """The oracle and oracle/sanitize_driver.c in one program. sanitized: AddressSanitizer and
    UndefinedBehaviorSanitizer, runtimes linked statically, every report fatal; otherwise the
    oracle's ordinary flags. Returns the program's path."""
    exe = os.path.join(out_dir, "oracle_driver_sanitized" if sanitized else "oracle_driver_plain")
    if sanitized:
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                 "-static-libasan", "-static-libubsan"]
    else:
        flags = ["-O2"]
    cmd = ["gcc"] + flags + ["-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-Wall", "-Wextra", "-o", exe, SRC,
                             os.path.join(HERE, "sanitize_driver.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
