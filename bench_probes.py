"""Peak probes of libdwm_probe.so: streaming copy / fill / read and an fp32 MFMA loop.

Not part of the convolution path or of the library package: they sit beside bench.py.
`python bench_probes.py` prints what the box reaches; run under `rocprofv3 --pmc FETCH_SIZE`
(or WRITE_SIZE) the copy of a known size (256 MiB read + 256 MiB written per launch)
calibrates those counters.  `python bench_probes.py build` compiles bench_probes.hip into
libdwm_probe.so next to this file (hipcc, gfx950; no GPU needed).
"""
import ctypes
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_P = ctypes.c_void_p
PROBE_LIB = os.path.join(_HERE, "libdwm_probe.so")


def build():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = PROBE_LIB + ".%d.tmp" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-x", "hip",
           os.path.join(_HERE, "bench_probes.hip"), "-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    os.replace(tmp, PROBE_LIB)
    return PROBE_LIB


def lib():
    path = PROBE_LIB
    if not os.path.exists(path):
        raise ImportError("libdwm_probe.so is not built: run `python bench_probes.py build`")
    L = ctypes.CDLL(path)
    L.dwm_probe_copy.argtypes = [_P, _P, ctypes.c_size_t, ctypes.c_int, _P]
    L.dwm_probe_fill.argtypes = [_P, ctypes.c_size_t, ctypes.c_int, _P]
    L.dwm_probe_read.argtypes = [_P, _P, ctypes.c_size_t, ctypes.c_int, _P]
    L.dwm_probe_mfma.argtypes = [_P, ctypes.c_int, ctypes.c_int, _P]
    return L


def measure(mib=256, reps=10, blocks=4096):
    """{'copy_GBps', 'fill_GBps', 'read_GBps', 'mfma_f32_TFLOPs'} measured with HIP events."""
    import torch
    L = lib()
    st = torch.cuda.current_stream().cuda_stream
    nbytes = mib << 20
    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
    b = torch.empty_like(a)
    o = torch.zeros(256, dtype=torch.float32, device="cuda")

    def timed(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    iters = 4000
    return {
        "bytes_per_launch": nbytes,
        "copy_GBps": 2 * nbytes / timed(lambda: L.dwm_probe_copy(a.data_ptr(), b.data_ptr(), nbytes, blocks, st)) / 1e6,
        "fill_GBps": nbytes / timed(lambda: L.dwm_probe_fill(b.data_ptr(), nbytes, blocks, st)) / 1e6,
        "read_GBps": nbytes / timed(lambda: L.dwm_probe_read(a.data_ptr(), o.data_ptr(), nbytes, blocks, st)) / 1e6,
        "mfma_f32_TFLOPs": 512 * 4 * iters * 4 * 4096 / timed(lambda: L.dwm_probe_mfma(o.data_ptr(), 512, iters, st)) / 1e9,
    }


if __name__ == "__main__":
    import json
    if sys.argv[1:2] == ["build"]:
        print(build())
        sys.exit(0)
    print(json.dumps(measure(int(sys.argv[1]) if len(sys.argv) > 1 else 256)))
