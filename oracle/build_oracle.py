"""Compile the C oracle into oracle/libgwq_oracle.so with gcc (no GPU code involved)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gwq_oracle.c")
LIB = os.path.join(HERE, "libgwq_oracle.so")


# With GWQ_ORACLE_SANITIZE=1 in the environment the oracle is built (into a library of its own) with gcc's address
# and undefined-behaviour sanitizers, every report fatal.  The Python that loads it must have the sanitizer runtime
# loaded first:  LD_PRELOAD="$(gcc -print-file-name=libasan.so):$LD_PRELOAD" ASAN_OPTIONS=detect_leaks=0
#                GWQ_ORACLE_SANITIZE=1 python -m pytest tests/test_oracle_pins.py -q
SANITIZE = os.environ.get("GWQ_ORACLE_SANITIZE", "") == "1"
if SANITIZE:
    LIB = os.path.join(HERE, "libgwq_oracle_san.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if SANITIZE else ["-O2"]
    cmd = ["gcc", *flags, "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
