"""Build libmaxscore.so for gfx950 with hipcc (cross-compiles without a GPU).

Every source is compiled to an object file under `_build/` (in parallel) and the objects are linked into one
shared library beside this file.  `build()` compiles everything; `build(incremental=True)` skips sources whose
object is newer than the source and every header.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build", "maxscore")
LIB = os.path.join(HERE, "libmaxscore.so")
SOURCES = ["api.cpp", "solver.hip", "softtopk.hip", "dispatch.hip", "movement.hip", "iter.hip", "training.hip",
           "operators.hip", "alg1.hip", "sinkhorn.hip", "gemm.hip", "noalloc.hip", "finish.hip", "oversub.hip"]


def _flags():
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC] + os.environ.get("MAXSCORE_CXXFLAGS", "").split()


def build(verbose: bool = False, incremental: bool = False, jobs: int = 8) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    newest_header = max(os.path.getmtime(h) for h in headers)
    flags = _flags()
    stamp = os.path.join(OBJ, "flags.txt")
    if incremental and (not os.path.exists(stamp) or open(stamp).read() != " ".join(flags)):
        incremental = False
    todo, objs = [], []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, s + ".o")
        objs.append(obj)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        todo.append([hipcc] + flags + ["-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        text = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        return r.returncode, text

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        results = list(ex.map(run, todo))
    for (rc, text), cmd in zip(results, todo):
        if text.strip():
            print(text, file=sys.stderr)
        if rc != 0:
            raise subprocess.CalledProcessError(rc, cmd)
    with open(stamp, "w") as f:
        f.write(" ".join(flags))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, incremental="--incremental" in sys.argv))
