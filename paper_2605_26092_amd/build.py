"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgoq.so")

# per-file extras: the GEMV's leading scalar kernel arguments arrive in scalar registers
EXTRA = {"goq_gemv.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=9"]}

FLAGS = ["-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
         # packed fp32 VALU forms are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(force: bool = True, extra=()) -> str:
    srcs = sources()
    deps = srcs + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "goq.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in srcs:
        obj = os.path.join(HERE, "_build", os.path.basename(src) + ".o")
        cmd = (["hipcc", "-c"] + [f for f in FLAGS if f != "-shared"] + EXTRA.get(os.path.basename(src), [])
               + list(extra) + ["-o", obj, src])
        procs.append((src, subprocess.Popen(cmd)))
        objs.append(obj)
    for src, p in procs:
        if p.wait() != 0:
            raise RuntimeError("hipcc failed on " + src)
    subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
