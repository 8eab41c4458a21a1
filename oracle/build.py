"""Compile the C oracle with gcc into oracle/liboracle_dsattn.so.

Test infrastructure only: nothing on the product path builds or loads this.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "dsattn_oracle.c"), os.path.join(HERE, "groupnorm_oracle.c"),
        os.path.join(HERE, "tconv_oracle.c"), os.path.join(HERE, "linear_oracle.c")]
LIB = os.path.join(HERE, "liboracle_dsattn.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and \
            os.path.getmtime(LIB) >= max(os.path.getmtime(s) for s in SRCS):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, *SRCS, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
