"""Compile the CPU oracle (oracle/quartet_ref.c) into oracle/libquartet_ref.so.

Test infrastructure: building the checker is not using it.  Flags matter for the
definition: no FMA contraction, no fast-math, IEEE fp32 on SSE.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "quartet_ref.c")
LIB = os.path.join(HERE, "libquartet_ref.so")

FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
         "-fno-fast-math", "-Wall", "-Wextra"]


SANITIZE = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (CPU only), for the tests' sanitizer leg."""
    flags = [f for f in FLAGS if f != "-O2"] + SANITIZE
    subprocess.run(["gcc"] + flags + [SRC, "-o", out_path, "-lm"], check=True)
    return out_path


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc"] + FLAGS + [SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
