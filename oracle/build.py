"""Compile the C oracle into oracle/libsparq_oracle.so with gcc (no HIP, no GPU).

`sanitize=True` builds a second library, libsparq_oracle_san.so, with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only); the pins are re-run against it by tests/test_oracle_sanitized.py.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sparq_oracle.c")
LIB = os.path.join(HERE, "libsparq_oracle.so")
LIB_SAN = os.path.join(HERE, "libsparq_oracle_san.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"] \
        if sanitize else ["-O2"]
    cmd = ["gcc"] + opt + ["-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra",
                           "-shared", "-fPIC", SRC, "-o", lib, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, sanitize="--sanitize" in sys.argv))
