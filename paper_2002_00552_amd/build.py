"""Build libdwm.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdwm.so")
PROBE_LIB = os.path.join(HERE, "libdwm_probe.so")
SOURCES = ["plan.cpp", "transforms.hip", "contract.hip", "fused.hip", "contract_batch.hip", "backward.hip", "wgrad.hip", "half.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    if not os.path.exists(PROBE_LIB):
        return True
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "dwm.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False):
    """Compile every HIP/C++ source into paper_2002_00552_amd/libdwm.so."""
    if not force and not stale():
        return LIB
    tmp = LIB + ".%d.tmp" % os.getpid()
    cmd = [HIPCC] + FLAGS + ["-x", "hip"] + sources() + ["-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    # the peak probes (streaming copy / fill / read, fp32 MFMA loop) live in a library of their own
    tmp = PROBE_LIB + ".%d.tmp" % os.getpid()
    cmd = [HIPCC] + FLAGS + ["-x", "hip", os.path.join(CSRC, "probe.hip"), "-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    os.replace(tmp, PROBE_LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
