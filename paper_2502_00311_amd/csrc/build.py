"""Build libsgc.so (HIP, gfx950) in-tree with hipcc. Usage: python build.py [--force]"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["api.hip", "topk.hip", "project.hip", "adam.hip", "apply.hip", "matrix.hip", "omp.hip", "omp_corr.hip", "omp_recur.hip", "outer.hip", "refresh.hip", "profile.hip", "probe.hip"]
LIB = os.path.join(HERE, "libsgc.so")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _newest_header():
    hs = [os.path.join(HERE, f) for f in os.listdir(HERE) if f.endswith(".h")]
    hs.append(os.path.join(HERE, "..", "..", "include", "sgc.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(src, force):
    obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
    path = os.path.join(HERE, src)
    if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), _newest_header()):
        return obj
    subprocess.check_call(["hipcc", *FLAGS, "-c", path, "-o", obj])
    return obj


def build(force=False):
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs, "-ldl"])
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
