"""Build libdwm.so in-tree with hipcc for gfx950 (cross-compiles without a GPU).

Every source is compiled to an object of its own (in parallel, objects kept under _build/) and
the objects are linked into paper_2002_00552_amd/libdwm.so.  build(force=True) recompiles
everything; build(force=False) only what is older than its sources.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdwm.so")
SOURCES = ["plan.cpp", "setup.cpp", "transforms.hip", "contract.hip", "fused.hip", "contract_batch.hip",
           "backward.hip", "backward_small.hip", "wgrad.hip", "half.hip", "bf16.hip", "noalloc.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
JOBS = min(8, os.cpu_count() or 1)


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]


def _headers():
    return [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h", ".inc"))] + [
        os.path.join(HERE, "..", "include", "dwm.h")]


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    return out


def _compile(src, force):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    if not force and os.path.exists(obj):
        t = os.path.getmtime(obj)
        if all(os.path.getmtime(d) <= t for d in [src] + _headers()):
            return obj, ""
    tmp = obj + ".%d.tmp" % os.getpid()
    out = _run([HIPCC] + FLAGS + ["-x", "hip", "-c", src, "-o", tmp])
    os.replace(tmp, obj)
    return obj, out


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in sources() + _headers())


def build(force=True, verbose=False):
    """Compile every HIP/C++ source and link paper_2002_00552_amd/libdwm.so."""
    if not force and not stale():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(JOBS) as ex:
        results = list(ex.map(lambda s: _compile(s, force), sources()))
    if verbose:
        for _, out in results:
            if out.strip():
                print(out)
    tmp = LIB + ".%d.tmp" % os.getpid()
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + [o for o, _ in results] + ["-o", tmp])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=False, verbose=True))
