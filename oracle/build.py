"""TEST INFRASTRUCTURE -- compiles the C oracle with gcc into oracle/_build/liboracle.so.

Building the checker is not using it: `__graft_entry__.build()` calls this so
that the GPU machine (which never compiles anything) finds the library in-tree.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "syrk_cholesky_oracle.c")
OUT_DIR = os.path.join(HERE, "lib")
OUT = os.path.join(OUT_DIR, "liboracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    os.makedirs(OUT_DIR, exist_ok=True)
    # -ffp-contract=off: no fused multiply-add, so every product and every sum
    # is rounded separately as the plain loops say.  No -march=native: the
    # library is built in one container and run on another machine.
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-o", OUT, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build())
