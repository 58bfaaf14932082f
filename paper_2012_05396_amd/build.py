"""Build libssd.so (HIP, gfx950 only) in-tree with hipcc.

The fused kernel is compiled once per worker count K = 1..16 (so that its
worker loops unroll) and per element type of the gradient buffers; the
objects are built in parallel and linked into one
shared library next to this file.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libssd.so")
MAX_K = 16
GRAD_DTYPES = 3  # binary32, bfloat16, binary16 gradient buffers

# -ffp-contract=off: one rounding per written operation (the rounding sequence
# is part of the library's contract).  Packed FP32 instructions stay off.
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument",
         # leading kernel arguments arrive in SGPRs at wave launch
         "-mllvm", "-amdgpu-kernarg-preload-count=14"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True)
    out = "\n".join(l for l in r.stdout.splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(jobs=None, verbose=False, defines=(), lib=None, obj_dir=None):
    """Compile every source and link libssd.so.  Always recompiles.
    `defines` ("-DX=1", ...), `lib` and `obj_dir` build an experimental
    variant elsewhere."""
    OBJ = obj_dir or globals()["OBJ"]
    LIB = lib or globals()["LIB"]
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    units = []
    for gd in range(GRAD_DTYPES):
        for k in range(1, MAX_K + 1):
            units.append((os.path.join(CSRC, "ssd_fused.hip"),
                          os.path.join(OBJ, "ssd_fused_g%d_k%d.o" % (gd, k)),
                          ["-DSSD_K=%d" % k, "-DSSD_GD=%d" % gd]))
    units.append((os.path.join(CSRC, "ssd_aux.hip"),
                  os.path.join(OBJ, "ssd_aux.o"), []))
    units.append((os.path.join(CSRC, "ssd_noalloc.hip"),
                  os.path.join(OBJ, "ssd_noalloc.o"), []))
    units.append((os.path.join(CSRC, "ssd_host.hip"),
                  os.path.join(OBJ, "ssd_host.o"), []))

    def one(u):
        src, obj, extra = u
        return _run(["hipcc"] + FLAGS + list(defines) + extra + ["-c", src, "-o", obj])

    with ThreadPoolExecutor(jobs) as ex:
        for msg in ex.map(one, units):
            if verbose and msg:
                print(msg)
    tmp = LIB + ".tmp%d" % os.getpid()
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] +
         [u[1] for u in units])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
