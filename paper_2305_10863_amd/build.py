"""Build libqv.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqv.so")
SOURCES = ["ctx.hip", "sample.hip", "gather.hip", "metrics.hip", "transpose.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def build(force=True, jobs=5):
    """Compile every source to an object (in parallel), then link."""
    objs, procs = [], []
    hdrs = [os.path.join(CSRC, "qv_internal.hpp"), os.path.join(HERE, "..", "include", "qv.h")]
    newest_hdr = max(os.path.getmtime(h) for h in hdrs)
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(CSRC, src.replace(".hip", ".o"))
        objs.append(o)
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), newest_hdr):
            procs.append((src, subprocess.Popen(["hipcc", *FLAGS, "-c", s, "-o", o])))
            if len(procs) >= jobs:
                name, p = procs.pop(0)
                if p.wait() != 0:
                    raise RuntimeError("hipcc failed on " + name)
    for name, p in procs:
        if p.wait() != 0:
            raise RuntimeError("hipcc failed on " + name)
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    write_build_info()
    return LIB


def write_build_info():
    """Beside the library: the commit it was built from, for runs on a copy of the tree without history."""
    import json
    root = os.path.join(HERE, "..")
    info = {"git": None, "dirty": None}
    try:
        info["git"] = subprocess.check_output(["git", "-C", root, "rev-parse", "--short", "HEAD"],
                                              stderr=subprocess.DEVNULL).decode().strip()
        info["dirty"] = bool(subprocess.check_output(["git", "-C", root, "status", "--porcelain", "--untracked-files=no"],
                                                     stderr=subprocess.DEVNULL).decode().strip())
    except Exception:
        pass
    with open(os.path.join(HERE, "build_info.json"), "w") as f:
        json.dump(info, f)


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
