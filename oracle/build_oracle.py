"""Compile the CPU oracle (test infrastructure) into oracle/libmodet_oracle.so with g++."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "modet_oracle.cpp")
LIB = os.path.join(HERE, "libmodet_oracle.so")
# another build of the same source (the sanitizer run of tests/test_sanitizers.py); never rebuilt from here
OVERRIDE = os.environ.get("MODET_ORACLE_LIBRARY")


def build(force: bool = True) -> str:
    if OVERRIDE:
        return OVERRIDE
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(True))
    sys.exit(0)
