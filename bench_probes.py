"""Peak probes of libdwm_probe.so: streaming copy / fill / read, an fp32 MFMA loop and an operand-delivery probe
(`python bench_probes.py mix`).

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
    L.dwm_probe_mix.argtypes = [_P, _P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint, ctypes.c_uint, _P]
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


def measure_mix(blocks=196, iters=2000):
    """Cycles (at a nominal 2.4 GHz) per iteration of the operand-delivery probe: one chunk's instruction mix of a
    16-bit contraction workgroup (4 MFMAs 32x32x16, 8 KB of LDS reads and 3 KB of global->LDS DMA per wave, eight
    waves per CU), each ingredient alone and together; DMA sources in L2 (one region shared by every workgroup) or
    with the third instruction streaming from memory (8 KB per iteration, shared by two workgroups of one XCD)."""
    import torch
    L = lib()
    st = torch.cuda.current_stream().cuda_stream
    src = torch.ones((1 << 26) + (1 << 31) + (1 << 20), dtype=torch.uint8, device="cuda")
    out = torch.zeros(256 * 512, dtype=torch.int32, device="cuda")
    res = {"blocks": blocks, "iters": iters}

    def run(name, mode, pair_stride, shared_mask):
        if L.dwm_probe_mix(src.data_ptr(), out.data_ptr(), mode, 16, blocks, pair_stride, shared_mask, st):
            raise RuntimeError("probe refused")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if L.dwm_probe_mix(src.data_ptr(), out.data_ptr(), mode, iters, blocks, pair_stride, shared_mask, st):
            raise RuntimeError("probe refused")
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(e0.elapsed_time(e1) * 1e-3 * 2.4e9 / iters, 1)

    m16 = (1 << 24) - 1
    run("mfma_only_clk", 0, 0, m16)
    run("lds_reads_only_clk", 1, 0, m16)
    run("dma_l2_only_clk", 2, 0, (1 << 20) - 1)
    run("dma_l2_16MB_only_clk", 2, 0, m16)
    run("dma_l2_plus_stream_only_clk", 2, 1 << 24, m16)
    run("all_l2_clk", 3, 0, m16)
    run("all_l2_plus_stream_clk", 3, 1 << 24, m16)
    run("all_l2_plus_stream_ring4_clk", 4, 1 << 24, m16)
    res["dma_l2_B_per_clk_per_CU"] = round(8 * 3 * 1024 / res["dma_l2_only_clk"], 1)
    res["lds_read_B_per_clk_per_CU"] = round(8 * 8 * 1024 / res["lds_reads_only_clk"], 1)
    res["mfma_clk_each"] = round(res["mfma_only_clk"] / 8, 1)
    return res


if __name__ == "__main__":
    import json
    if sys.argv[1:2] == ["build"]:
        print(build())
        sys.exit(0)
    if sys.argv[1:2] == ["mix"]:
        print(json.dumps(measure_mix(int(sys.argv[2]) if len(sys.argv) > 2 else 196)))
        sys.exit(0)
    print(json.dumps(measure(int(sys.argv[1]) if len(sys.argv) > 1 else 256)))
