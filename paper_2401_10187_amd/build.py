"""Compile the HIP library for gfx950 into paper_2401_10187_amd/libkronmatmul.so (in-tree).

The kernel instances are spread over one translation unit per kernel family (csrc/inst_*.hip) so that
they compile side by side; csrc/kronmatmul.hip holds the C-ABI, the planner and the two kernels
without compile-time shapes."""
import glob
import os
import subprocess
import time
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkronmatmul.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep hipcc from forming packed-fp32 instructions out of ordinary float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    t0 = time.time()
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose:
        print("%.0f s: %s" % (time.time() - t0, os.path.basename(cmd[-1])), flush=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, flush=True)


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _stale(obj):
    """True unless `obj` is newer than every file its dependency list (written by -MD) names."""
    dep = obj[:-2] + ".d"
    if not (os.path.exists(obj) and os.path.exists(dep)):
        return True
    names = open(dep).read().replace("\\\n", " ").split(":", 1)[1].split()
    t = os.path.getmtime(obj)
    return any(not os.path.exists(n) or os.path.getmtime(n) > t for n in names)


def build(verbose=False, jobs=None, incremental=False):
    """Recompiles every translation unit (with incremental=True only those whose sources changed, a
    convenience while working on one kernel); returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJ, os.path.basename(s)[:-4] + ".o") for s in srcs]
    todo = [(s, o) for s, o in zip(srcs, objs) if not incremental or _stale(o)]
    jobs = jobs or min(max(len(todo), 1), os.cpu_count() or 1, 16)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda so: _run([hipcc] + HIPCC_FLAGS + ["-MD", "-MF", so[1][:-2] + ".d", "-c", "-o", so[1], so[0]],
                                      verbose), todo))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, verbose)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv[1:]))
