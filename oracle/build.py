"""Compile the CPU oracle (test infrastructure) with gcc.

Two shared objects are built from the one source file: binary64 (the plain
oracle) and binary32 with contraction off (the GPU-order oracle).
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ssd_oracle.c")
FLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
         "-shared", "-fPIC"]
VARIANTS = {"f32": "float", "f64": "double"}


def lib_path(sfx):
    return os.path.join(HERE, "libssd_oracle_%s.so" % sfx)


def build(force=False):
    """Build both variants; returns {suffix: path}."""
    out = {}
    for sfx, real in VARIANTS.items():
        dst = lib_path(sfx)
        stale = (not os.path.exists(dst)
                 or os.path.getmtime(dst) < os.path.getmtime(SRC))
        if force or stale:
            tmp = dst + ".tmp%d" % os.getpid()
            subprocess.check_call(["gcc"] + FLAGS +
                                  ["-DREAL=" + real, "-DSFX=" + sfx, SRC,
                                   "-o", tmp])
            os.replace(tmp, dst)
        out[sfx] = dst
    return out


if __name__ == "__main__":
    print(build(force=True))
