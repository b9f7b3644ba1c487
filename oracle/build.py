"""Compile the oracle (test infrastructure, CPU only) into oracle/liboracle.so.

Plain g++ -O2, no -ffast-math and no FMA contraction, so the arithmetic is the
one written in the source.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "augur_oracle.cpp")
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


SAN_LIB = os.path.join(HERE, "liboracle_sanitized.so")


def build_sanitized() -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (CPU only), for the
    test that runs the small sweeps under them; a finding aborts the process."""
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fPIC", "-shared",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-o", SAN_LIB, SRC]
    subprocess.run(cmd, check=True)
    return SAN_LIB


if __name__ == "__main__":
    print(build())
