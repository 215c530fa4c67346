"""Compile the CPU oracle (test infrastructure) into oracle/libsol_oracle.so with gcc.

build(sanitize=True) makes a second library, oracle/libsol_oracle_san.so, with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only); tests/test_oracle_sanitizers.py runs the oracle's entry points
through it in a child process."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libsol_oracle.so")
LIB_SAN = os.path.join(HERE, "libsol_oracle_san.so")
SRC = os.path.join(HERE, "sol_oracle.c")
DEPS = (SRC, os.path.join(HERE, "sol_oracle.h"))


def build(force: bool = True, sanitize: bool = False) -> str:
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= max(os.path.getmtime(p) for p in DEPS):
        return lib
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"] \
        if sanitize else ["-O2"]
    cmd = ["gcc"] + flags + ["-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                             "-Wall", "-Wextra", "-o", lib, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build())
