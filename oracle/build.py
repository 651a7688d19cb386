"""Compile the C oracle into two shared objects (fp32 loops and fp64 loops).

Test infrastructure: run by the build entry point and, if the objects are missing or
older than the source, by the loader in this package.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fastkv_oracle.c")
LIBS = {"f32": os.path.join(HERE, "liboracle_f32.so"), "f64": os.path.join(HERE, "liboracle_f64.so")}
CFLAGS = ["-O2", "-fPIC", "-shared", "-fopenmp", "-std=c11", "-Wall", "-Wextra"]


def build(force: bool = False) -> dict:
    for prec, out in LIBS.items():
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        cmd = ["gcc", *CFLAGS, *(["-DORC_F64"] if prec == "f64" else []), SRC, "-o", out + ".tmp", "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(out + ".tmp", out)
    return dict(LIBS)


if __name__ == "__main__":
    print(build(force=True))
