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


SAN_LIB = os.path.join(HERE, "libfs_oracle_san.so")
SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def build(force: bool = True, sanitize: bool = False) -> str:
    """sanitize=True: a second library, libfs_oracle_san.so, instrumented with the address and undefined-behaviour
    sanitizers (host code only); the ordinary one is left as it is."""
    lib = SAN_LIB if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    tag = "_san" if sanitize else ""
    flags = [f for f in CFLAGS if f != "-O2"] + SAN_FLAGS if sanitize else CFLAGS
    o32 = os.path.join(HERE, f"fs_oracle_f32{tag}.o")
    o64 = os.path.join(HERE, f"fs_oracle_f64{tag}.o")
    subprocess.check_call(["gcc", *flags, "-DORC_F32", "-c", SRC, "-o", o32])
    subprocess.check_call(["gcc", *flags, "-c", SRC, "-o", o64])
    subprocess.check_call(["gcc", "-shared", "-fopenmp", *(SAN_FLAGS[:1] if sanitize else []), o32, o64, "-lm", "-o", lib])
    os.remove(o32)
    os.remove(o64)
    return lib


if __name__ == "__main__":
    print(build())
