"""Compile the float64 C oracle into oracle/liblora_oracle.so (gcc, OpenMP).

Test infrastructure: building the checker is not using it.
`-ffp-contract=off` keeps every multiply and add separately rounded, so the
bitwise statements made in the oracle's tests hold on any x86-64 host.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lora_oracle.c")
OUT = os.path.join(HERE, "liblora_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-O3", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", OUT, SRC]
    subprocess.check_call(cmd)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
