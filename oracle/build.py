"""Compile the fp64 CPU oracle (test infrastructure) into oracle/liboracle.so with gcc.

A second configuration, liboracle_ubsan.so, is the same source built with the undefined-behaviour sanitizer (its
runtime linked in statically, every report fatal) and stricter warnings; the CPU test suite runs the oracle's pins
under it once.  oracle/san_check.c, linked against the same source with AddressSanitizer + UBSan into the executable
oracle/san_check, walks the entry points over edge shapes (see tests/test_oracle_sanitized.py)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bimamba_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
LIB_UBSAN = os.path.join(HERE, "liboracle_ubsan.so")
SAN_SRC = os.path.join(HERE, "san_check.c")
SAN_EXE = os.path.join(HERE, "san_check")
SAN_PLAIN = os.path.join(HERE, "san_check_plain")
COMMON = ["-std=c99", "-fopenmp", "-Wall", "-Wextra", "-ffp-contract=off"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    subprocess.run(["gcc", "-O2", "-fPIC", "-shared"] + COMMON + ["-o", LIB, SRC, "-lm"], check=True)
    return LIB


def build_sanitized(force: bool = False):
    """(liboracle_ubsan.so, san_check, san_check_plain): built on demand by the CPU tests; returns the three paths."""
    newest = max(os.path.getmtime(SRC), os.path.getmtime(SAN_SRC))
    if force or not os.path.exists(LIB_UBSAN) or os.path.getmtime(LIB_UBSAN) < os.path.getmtime(SRC):
        subprocess.run(["gcc", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=undefined,float-divide-by-zero",
                        "-fno-sanitize-recover=all", "-static-libubsan"] + COMMON + ["-o", LIB_UBSAN, SRC, "-lm"], check=True)
    if force or not os.path.exists(SAN_EXE) or os.path.getmtime(SAN_EXE) < newest:
        subprocess.run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        "-fno-omit-frame-pointer", "-static-libasan"] + COMMON + ["-o", SAN_EXE, SAN_SRC, SRC, "-lm"], check=True)
    if force or not os.path.exists(SAN_PLAIN) or os.path.getmtime(SAN_PLAIN) < newest:
        subprocess.run(["gcc", "-O2"] + COMMON + ["-o", SAN_PLAIN, SAN_SRC, SRC, "-lm"], check=True)   # same walk, regular flags
    return LIB_UBSAN, SAN_EXE, SAN_PLAIN


if __name__ == "__main__":
    print(build())
