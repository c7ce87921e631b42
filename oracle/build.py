"""Compile the oracle's C part (plain gcc, OpenMP) into oracle/liblpref.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lpref.c")
LIB = os.path.join(HERE, "liblpref.so")


def build(force: bool = True) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra", SRC, "-o", LIB]
        subprocess.run(cmd, check=True)
    return LIB


def build_selfcheck() -> str:
    """The oracle's C part under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): compiles
    lpref_selfcheck.c, which includes lpref.c, into an executable that drives every routine over small ragged shapes.
    Returns its path; running it must print 0 failures and exit 0."""
    exe = os.path.join(HERE, "lpref_selfcheck")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-std=c99", "-Wall", "-Wextra", os.path.join(HERE, "lpref_selfcheck.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build())
