"""Compiles the CPU oracle (test infrastructure) into oracle/liboracle.so.

`python -m oracle.build --sanitize` (or build_sanitized()) instead compiles the oracle's
sources together with oracle/sanitize_driver.cpp into the program oracle/oracle_sanitized
with AddressSanitizer and UndefinedBehaviorSanitizer; running it exercises every entry
point on a 256-configuration space, without Python in the process."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, f) for f in ("tuner_oracle.cpp", "train_oracle.cpp")]
LIB_PATH = os.path.join(HERE, "liboracle.so")
SANITIZED_PATH = os.path.join(HERE, "oracle_sanitized")


def build(verbose: bool = False) -> str:
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread",
           "-ffp-contract=off", "-o", LIB_PATH, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


def build_sanitized(verbose: bool = False) -> str:
    """The sanitizer runtimes are linked statically, so that the program does not depend on
    the order in which shared libraries are loaded into the process."""
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-pthread", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-static-libasan", "-static-libubsan",
           "-o", SANITIZED_PATH, *SOURCES, os.path.join(HERE, "sanitize_driver.cpp")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return SANITIZED_PATH


if __name__ == "__main__":
    if "--sanitize" in sys.argv[1:]:
        build_sanitized(verbose=True)
    else:
        build(verbose=True)
