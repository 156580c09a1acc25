"""Compile the CPU oracle (test infrastructure) into oracle/libpetals_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "petals_oracle.c")
LIB = os.path.join(HERE, "libpetals_oracle.so")

# -O2, no fast-math, no FMA contraction: the fp32 expressions that decide int8
# codes must evaluate exactly as written.
CMD = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
       "-shared", "-fPIC", SRC, "-o", LIB, "-lm"]


def build(force=True):
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(CMD)
    return LIB


SELFCHECK = os.path.join(HERE, "selfcheck_san")


def build_selfcheck():
    """The oracle and its driver (selfcheck.c) as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer; running it exits non-zero on any report."""
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra",
           SRC, os.path.join(HERE, "selfcheck.c"), "-o", SELFCHECK, "-lm"]
    subprocess.check_call(cmd)
    return SELFCHECK


if __name__ == "__main__":
    print(build())
