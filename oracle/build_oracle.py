"""Compile the plain-C oracle into ``oracle/libmglu_oracle.so`` with gcc.

Test infrastructure: building the checker is not using it.  Run as a script
(``python oracle/build_oracle.py``) or call :func:`build`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mglu_oracle.c")
LIB = os.path.join(HERE, "libmglu_oracle.so")


def build(force=True):
    """Compile the oracle; with ``force=False`` only when the library is absent or stale."""
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
           "-Wall", "-Wextra", "-o", tmp, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
