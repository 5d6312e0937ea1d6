"""Compiles the C oracle (``slim_oracle.c``) into ``libslim_oracle.so`` beside it."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "slim_oracle.c")
LIB = os.path.join(HERE, "libslim_oracle.so")


def build(force: bool = True) -> str:
    """gcc -O2 -fopenmp, never -ffast-math (the quantiser needs IEEE fp32 division)."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
           "-fno-fast-math", "-ffp-contract=off", "-o", tmp, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
