"""Builds libfreeride.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfreeride.so")
SOURCES = ["runtime.cpp", "stage.cpp", "pagerank.hip", "pagerank_prep.hip", "sgd.hip", "gemm.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-pthread",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # keep packed-fp32 instructions out
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "common.h"), os.path.join(CSRC, "pr_layout.h"),
                        os.path.join(ROOT, "include", "freeride.h"),
                        os.path.join(ROOT, "include", "freeride_device.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True) -> str:
    """Compile every source into one shared library; returns its path."""
    if not force and not is_stale():
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs, procs = [], []
    for src in sources():                      # one hipcc per source, all at once, then one link
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        procs.append(subprocess.Popen([HIPCC] + FLAGS + ["-x", "hip", "-c", src, "-o", obj]))
    failed = [p.args for p in procs if p.wait() != 0]
    if failed:
        raise RuntimeError("hipcc failed: %s" % " ".join(failed[0]))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread"] + objs + ["-o", tmp])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
