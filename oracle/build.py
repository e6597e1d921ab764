"""Compile the C oracle (test infrastructure) into two shared objects beside this
file: liborc64.so (real = double, the parity authority) and liborc32.so (the same
text with real = float)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "drf_oracle.c")
FLAGS = ["-O3", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra"]


def lib_path(bits):
    return os.path.join(HERE, "liborc%d.so" % bits)


def build(force=False):
    for bits, extra in ((64, []), (32, ["-DORC_F32"])):
        out = lib_path(bits)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        subprocess.check_call(["gcc", *FLAGS, *extra, SRC, "-o", out, "-lm"])


if __name__ == "__main__":
    build(force=True)
    print("built", lib_path(64), lib_path(32))
