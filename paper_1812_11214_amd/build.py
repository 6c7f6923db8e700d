"""Compile the HIP library in-tree: csrc/*.{hip,cpp} -> libscat.so (gfx950).

Every source becomes one object under _build/ (compiled in parallel), then one link step.
`build()` recompiles everything; `build(incremental=True)` only the sources that are newer
than their object (any header change rebuilds all)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libscat.so")
SOURCES = ("scat_host.cpp", "scat_host3d.cpp", "scat_kernels.hip", "scat_tree.hip", "scat_node.hip",
           "scat_backward.hip", "scat_3d.hip", "scat_capi.hip")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _stale(src, obj, newest_header):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return os.path.getmtime(src) > t or newest_header > t


def build(verbose=False, incremental=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
    headers.append(os.path.join(HERE, "..", "include", "scat.h"))
    newest = max(os.path.getmtime(h) for h in headers if os.path.exists(h))
    jobs = []
    objs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        if not incremental or _stale(src, obj, newest):
            jobs.append([hipcc] + FLAGS + ["-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)

    workers = max(1, min(len(jobs), len(os.sched_getaffinity(0)), 16))
    with ThreadPoolExecutor(workers) as ex:
        for cmd, res in zip(jobs, ex.map(run, jobs)):
            out = "\n".join(l for l in res.stdout.splitlines()
                            if "packed-fp32-ops" not in l)  # the host pass does not know the feature
            if out.strip():
                print(out, flush=True)
            if res.returncode != 0:
                raise subprocess.CalledProcessError(res.returncode, cmd)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))
