"""Random small layers through every path of the library, each against the FP64 oracle.

The shapes are drawn from a seeded generator that mixes what the hand-picked cases of the other files fix one
at a time: kernels of 1..13 taps (square or not), strides 1..8 (also above the kernel size), paddings up to the
kernel size, few or many channels, images down to one pixel wide.  Every case runs the forward pass (the
planner's path and the staged path), the entry point that allocates nothing, the data gradient (both paths where
the single kernel applies), the filter gradient, and the binary16 and bfloat16 forward passes (staged and single
kernel) -- the first mismatch names the path and the shape.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2002_00552_amd as dwm
from dwm_gpu import Runner
from test_gpu_backward import BwdRunner, WgradRunner
from test_gpu_bf16 import Bf16Runner
from test_gpu_half import HalfRunner

pytestmark = pytest.mark.gpu

TOL, TOL16 = 1e-4, 2e-5


def _rel(a, ref):
    return float(np.max(np.abs(a.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def _draw(rng):
    R = int(rng.integers(1, 14))
    S = R if rng.random() < 0.6 else int(rng.integers(1, 14))
    s = int(rng.choice([1, 1, 2, 2, 3, 4, 5, 6, 8]))
    P = int(rng.integers(0, max(R, S) + 1))
    C = int(rng.integers(1, 9)) if rng.random() < 0.5 else int(rng.integers(9, 200))
    K = int(rng.integers(1, 300))
    big = rng.random() < 0.15
    H = int(rng.integers(max(1, R - 2 * P), 150 if big else 48))
    W = int(rng.integers(max(1, S - 2 * P), 150 if big else 48))
    N = int(rng.integers(1, 9))
    return N, C, H, W, K, R, S, s, P


def _check_layer(shape, rng):
    N, C, H, W, K, R, S, s, P = shape
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    dy = rng.uniform(-1, 1, (N, K, OH, OW)).astype(np.float32)
    ref = oracle.direct_f64(x, w, s, P)
    for staged in (False, True):
        r = Runner(*shape)
        try:
            if staged:
                dwm.dwm_plan_set_variant(r.plan, "forward", 0)
            r.set_filter(w)
            y = r.forward(x)
        finally:
            r.close()
        assert np.all(np.isfinite(y)) and _rel(y, ref) <= TOL, ("forward, staged" if staged else "forward", shape)
    # the entry point that allocates nothing: a plan of its own, no workspace handed over
    plan = dwm.dwm_plan_create(*shape)
    try:
        info = dwm.dwm_plan_info(plan)
        xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        U = torch.empty(max(dwm.dwm_plan_filter_bytes(plan) // 4, 1), dtype=torch.float32, device="cuda")
        yd = torch.full((N, K, info.OH, info.OW), float("nan"), dtype=torch.float32, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        dwm.dwm_filter_transform(plan, wd.data_ptr(), U.data_ptr(), st)
        if info.forward_path == 1 or dwm.dwm_plan_workspace_bytes(plan) <= dwm.dwm_static_scratch_bytes():
            dwm.dwm_conv_forward_static(plan, xd.data_ptr(), U.data_ptr(), yd.data_ptr(), st)
            torch.cuda.synchronize()
            y = yd.cpu().numpy()
            assert np.all(np.isfinite(y)) and _rel(y, ref) <= TOL, ("forward, no allocation", shape)
    finally:
        dwm.dwm_plan_destroy(plan)
    ref_dx = oracle.backward_data_f64(dy, w, (N, C, H, W), s, P)
    for path in (0, 1):
        try:
            b = BwdRunner(*shape, path=path)
        except dwm.DwmError:
            assert path == 1  # the single kernel does not apply to every layer
            continue
        try:
            dx = b.run(dy, w)
        finally:
            b.close()
        assert np.all(np.isfinite(dx)) and _rel(dx, ref_dx) <= TOL, ("data gradient, path %d" % path, shape)
    g = WgradRunner(*shape)
    try:
        dw = g.run(x, dy)
    finally:
        g.close()
    assert np.all(np.isfinite(dw)) and _rel(dw, oracle.backward_filter_f64(x, dy, (K, C, R, S), s, P)) <= TOL, \
        ("filter gradient", shape)
    x16, w16 = x.astype(np.float16), w.astype(np.float16)
    ref16 = oracle.dwm_half_f64(x16, w16, s, P)
    xb = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    wb = torch.from_numpy(w).to(torch.bfloat16).float().numpy()
    refb = oracle.dwm_bf16_f64(xb, wb, s, P)
    for name, cls, a, b_, r16 in (("binary16", HalfRunner, x16, w16, ref16), ("bfloat16", Bf16Runner, xb, wb, refb)):
        for forward in (0, 1):
            try:
                h = cls(*shape, forward=forward)
            except dwm.DwmError:
                assert forward == 1  # the single kernel does not apply to every layer
                continue
            try:
                y = h.run(a, b_, f32out=True)
            finally:
                h.close()
            assert np.all(np.isfinite(y)) and _rel(y, r16) <= TOL16, ("%s forward, form %d" % (name, forward), shape)


@pytest.mark.parametrize("seed", [7, 21, 1234])
def test_random_layers_every_path(seed):
    rng = np.random.default_rng(seed)
    done = 0
    while done < 60:
        shape = _draw(rng)
        N, C, H, W, K, R, S, s, P = shape
        if H + 2 * P < R or W + 2 * P < S or N * C * H * W * K * R * S > 2e10:
            continue
        print("layer", shape, flush=True)
        _check_layer(shape, rng)
        done += 1


def _draw_medium(rng):
    R = int(rng.choice([1, 2, 3, 3, 4, 5, 5, 7, 7, 9, 11]))
    S = R if rng.random() < 0.8 else int(rng.choice([1, 3, 5, 7]))
    s = int(rng.choice([1, 1, 1, 2, 2, 3]))
    P = int(rng.integers(0, R // 2 + 2))
    C = int(rng.choice([24, 32, 48, 64, 64, 96, 128, 160, 256]))
    K = int(rng.choice([32, 64, 96, 128, 192, 256, 320]))
    return int(rng.integers(1, 40)), C, int(rng.integers(10, 64)), int(rng.integers(10, 64)), K, R, S, s, P


@pytest.mark.parametrize("seed", [5, 77])
def test_random_medium_layers_split_modes_variants_and_repeats(seed):
    """Layers of 40-4000 contraction tiles (many channels and filters) against sampled oracle outputs: the three
    ways of sharing out the tiles, a random contraction variant and input-transform form, twelve more launches
    through the same plan (bit-identical: split tiles are summed in a fixed order), the data gradient, the filter
    gradient on the smaller ones, and the binary16 path with random variants of its own."""
    rng = np.random.default_rng(seed)
    done = 0
    while done < 25:
        shape = _draw_medium(rng)
        N, C, H, W, K, R, S, s, P = shape
        if H + 2 * P < R or W + 2 * P < S:
            continue
        OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
        T = N * ((OH + 1) // 2) * ((OW + 1) // 2)
        tiles = ((K + 63) // 64) * ((T + 63) // 64)
        flops = 2.0 * N * K * C * R * S * OH * OW
        if tiles < 40 or tiles > 4000 or flops > 1.2e11:
            continue
        print("layer", shape, "tiles", tiles, flush=True)
        x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
        w = (rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)
        dy = rng.uniform(-1, 1, (N, K, OH, OW)).astype(np.float32)
        idx = rng.choice(N * K * OH * OW, min(N * K * OH * OW, 6000), replace=False)
        ref = oracle.direct_f64_at(x, w, s, P, idx)
        scale = np.max(np.abs(ref))
        for split in (0, 1, 2):
            r = Runner(*shape, variants={"split": split})
            try:
                r.set_filter(w)
                y = r.forward(x)
                if split == 0:
                    xs = torch.from_numpy(x).cuda()
                    for _ in range(12):
                        dwm.dwm_conv_forward(r.plan, xs.data_ptr(), r.Ugw.data_ptr(), r.y.data_ptr(), r.stream())
                    torch.cuda.synchronize()
                    assert np.array_equal(r.y.cpu().numpy(), y), ("repeated launches", shape)
            finally:
                r.close()
            assert np.all(np.isfinite(y)) and np.max(np.abs(y.ravel()[idx] - ref)) / scale <= TOL, ("split", split, shape)
        for _ in range(2):
            variants = {"contract": int(rng.integers(10, 20)), "input": int(rng.integers(0, 4))}
            try:
                r = Runner(*shape, variants=variants)
            except dwm.DwmError:
                continue  # a chunk depth or a staged region that does not fit this layer
            try:
                r.set_filter(w)
                y = r.forward(x)
            finally:
                r.close()
            assert np.all(np.isfinite(y)) and np.max(np.abs(y.ravel()[idx] - ref)) / scale <= TOL, (variants, shape)
        idx2 = rng.choice(N * C * H * W, min(N * C * H * W, 6000), replace=False)
        ref_dx = oracle.backward_data_f64_at(dy, w, (N, C, H, W), s, P, idx2)
        b = BwdRunner(*shape)
        try:
            dx = b.run(dy, w)
        finally:
            b.close()
        assert np.all(np.isfinite(dx))
        assert np.max(np.abs(dx.ravel()[idx2] - ref_dx)) / max(np.max(np.abs(ref_dx)), 1e-30) <= TOL, ("data gradient", shape)
        if flops <= 3e9:
            g = WgradRunner(*shape)
            try:
                dw = g.run(x, dy)
            finally:
                g.close()
            assert np.all(np.isfinite(dw)) and _rel(dw, oracle.backward_filter_f64(x, dy, (K, C, R, S), s, P)) <= TOL, \
                ("filter gradient", shape)
        x16, w16 = x.astype(np.float16), w.astype(np.float16)
        ref16 = oracle.direct_f64_at(x16.astype(np.float32), w16.astype(np.float32), s, P, idx)
        h = HalfRunner(*shape, forward=0)
        try:
            y0 = h.run(x16, w16, f32out=True)
        finally:
            h.close()
        # against the exact convolution of the 16-bit inputs: the band of the format
        assert np.all(np.isfinite(y0)) and np.max(np.abs(y0.ravel()[idx] - ref16)) / np.max(np.abs(ref16)) <= 3e-3, shape
        for _ in range(2):
            try:
                h = HalfRunner(*shape, forward=0, variant=int(rng.integers(30, 48)), input_variant=int(rng.integers(0, 2)))
            except dwm.DwmError:
                continue
            try:
                y = h.run(x16, w16, f32out=True)
            finally:
                h.close()
            assert np.max(np.abs(y - y0)) / np.max(np.abs(ref16)) <= TOL16, ("binary16 variant", shape)
        done += 1
