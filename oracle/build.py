"""Compile the float64 C oracle into oracle/libpsf_oracle.so (gcc, OpenMP over units).

Test infrastructure only: nothing in the product path imports this package.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "psf_oracle.c")
LIB = os.path.join(HERE, "libpsf_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


SAN_LIB = os.path.join(HERE, "libpsf_oracle_san.so")


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (host code only),
    for the test that runs the pin suite's cases through it.  A process that loads it needs
    the sanitizer runtime first in LD_PRELOAD (gcc -print-file-name=libasan.so)."""
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           SRC, "-o", SAN_LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return SAN_LIB


if __name__ == "__main__":
    print(build())
