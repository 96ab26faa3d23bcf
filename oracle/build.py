"""Compile the CPU oracle (test infrastructure) into oracle/libfs_oracle.so.

The single C source is compiled twice, once per precision, and linked into one library.
Run as `python oracle/build.py`; `__graft_entry__.build()` calls `build()` too.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fs_oracle.c")
LIB = os.path.join(HERE, "libfs_oracle.so")
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-fopenmp", "-ffp-contract=off", "-mfma", "-Wall", "-Wextra",
          "-Wno-unused-parameter"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    o32 = os.path.join(HERE, "fs_oracle_f32.o")
    o64 = os.path.join(HERE, "fs_oracle_f64.o")
    subprocess.check_call(["gcc", *CFLAGS, "-DORC_F32", "-c", SRC, "-o", o32])
    subprocess.check_call(["gcc", *CFLAGS, "-c", SRC, "-o", o64])
    subprocess.check_call(["gcc", "-shared", "-fopenmp", o32, o64, "-lm", "-o", LIB])
    os.remove(o32)
    os.remove(o64)
    return LIB


if __name__ == "__main__":
    print(build())
