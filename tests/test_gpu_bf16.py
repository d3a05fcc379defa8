"""GPU parity tests of the bfloat16 forward path (dwm_bf16_*), called through the C ABI,
against the FP64 oracle with bfloat16 storage (oracle.dwm_bf16_f64: x, w, U and V in bfloat16,
sums in FP64).  Host arrays are float32 arrays that hold bfloat16 values; torch converts them
(exactly) to device tensors of bfloat16 patterns and back.

Bars.
* Output left in FP32 (dwm_bf16_conv_forward_f32out): the GPU differs from the oracle only by the
  FP32 accumulation of exact products -- max |y - y_ref| <= 2e-5 * max |y_ref| (sums of up to a
  few thousand terms, each partial sum rounded to 2^-24 relative).
* Output in bfloat16 (dwm_bf16_conv_forward): after the last rounding both sides sit on the
  bfloat16 grid; an FP32 accumulation error can tip a value over a rounding boundary, so elements
  may differ by one bfloat16 step (plus the FP32-output bar itself where an output is so small
  that its step is below that bar), and only a small fraction of them may differ at all.
* Where every intermediate is exactly representable the result is the exact convolution, bit for
  bit; the closed forms that fix the oracle's rounding points are reproduced bit for bit too.
"""
import numpy as np
import pytest
import torch

import dwm_workloads as wl
import oracle
import paper_2002_00552_amd as dwm

pytestmark = pytest.mark.gpu

TOL_F32OUT = 2e-5


class Bf16Runner:
    def __init__(self, N, C, H, W, K, R, S, stride, pad, variant=None, input_variant=None, forward=0, classes=-1):
        # forward: 0 the staged path (what most tests here are about), 1 the single kernel, -1 the planner's choice
        self.plan = dwm.dwm_bf16_plan_create(N, C, H, W, K, R, S, stride, pad)
        dwm.dwm_bf16_set_variant(self.plan, "forward", forward)
        # classes: 0 the general single kernel, -1 the one built for the layer's list of classes where there is one
        dwm.dwm_bf16_set_variant(self.plan, "classes", classes)
        if variant is not None:
            dwm.dwm_bf16_set_variant(self.plan, "contract", variant)
        if input_variant is not None:
            dwm.dwm_bf16_set_variant(self.plan, "input", input_variant)
        self.info = dwm.dwm_bf16_plan_info(self.plan)
        dev = torch.device("cuda:0")
        nan16 = 0x7FC0
        self.U = torch.full((dwm.dwm_bf16_filter_bytes(self.plan) // 2,), nan16, dtype=torch.int16, device=dev)
        self.ws = torch.full((max(dwm.dwm_bf16_workspace_bytes(self.plan), 256),), 0xFF, dtype=torch.uint8, device=dev)
        dwm.dwm_bf16_set_workspace(self.plan, self.ws.data_ptr(), self.ws.numel())
        self.shape_y = (N, K, self.info.OH, self.info.OW)

    def run(self, x16, w16, f32out=False):
        st = torch.cuda.current_stream().cuda_stream
        x = torch.from_numpy(np.ascontiguousarray(x16, dtype=np.float32)).to(torch.bfloat16).cuda()
        w = torch.from_numpy(np.ascontiguousarray(w16, dtype=np.float32)).to(torch.bfloat16).cuda()
        assert torch.equal(x.float().cpu(), torch.from_numpy(np.ascontiguousarray(x16, dtype=np.float32)))
        dwm.dwm_bf16_filter_transform(self.plan, w.data_ptr(), self.U.data_ptr(), st)
        if f32out:
            y = torch.full(self.shape_y, float("nan"), dtype=torch.float32, device="cuda:0")
            dwm.dwm_bf16_conv_forward_f32out(self.plan, x.data_ptr(), self.U.data_ptr(), y.data_ptr(), st)
        else:
            y = torch.full(self.shape_y, float("nan"), dtype=torch.bfloat16, device="cuda:0")
            dwm.dwm_bf16_conv_forward(self.plan, x.data_ptr(), self.U.data_ptr(), y.data_ptr(), st)
        torch.cuda.synchronize()
        return y.float().cpu().numpy()

    def close(self):
        dwm.dwm_bf16_plan_destroy(self.plan)


def _rand16(N, C, H, W, K, R, S, s, P, seed, dist="uniform"):
    rng = np.random.default_rng(seed)
    if dist == "relu_normal":
        x = np.maximum(rng.standard_normal((N, C, H, W)), 0.0)
    elif dist == "normal":
        x = rng.standard_normal((N, C, H, W))
    else:
        x = rng.uniform(-1, 1, (N, C, H, W))
    w = rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))
    return _bf(x), _bf(w)


def _bf(a):
    """float32 array of the bfloat16 values nearest to a."""
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).float().numpy()


def _ulp16(v):
    """Spacing of bfloat16 at |v| (float64 array)."""
    a = np.maximum(np.abs(v), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def _check_half_out(y16, ref64):
    ref16 = oracle.round_bfloat16(ref64)
    got = y16.astype(np.float64)
    assert np.all(np.isfinite(got))
    diff = np.abs(got - ref16)
    step = np.maximum(_ulp16(got), _ulp16(ref16))
    # before the last rounding the two sides differ by at most delta (the FP32-output bar); the
    # rounding can turn that into one bfloat16 step, or, for outputs so small that a step is below
    # delta, into delta plus a step
    delta = TOL_F32OUT * float(np.max(np.abs(ref64)))
    assert np.all(diff <= step + delta), "beyond one bfloat16 step: %g" % float(np.max((diff - delta) / step))
    assert np.mean(diff > 0) < 0.02, "fraction of differing elements %g" % float(np.mean(diff > 0))


SHAPES = [  # N, C, H, W, K, R, S, stride, pad
    (1, 16, 32, 32, 16, 5, 5, 1, 2),     # benchmark config 1
    (2, 3, 13, 15, 5, 5, 5, 1, 2),       # C = 3: groups of eight rows straddle parts
    (3, 8, 19, 21, 70, 3, 3, 2, 1),      # stride 2, odd sizes, K over one tile
    (2, 24, 14, 14, 40, 7, 7, 1, 3),     # pieces 3,3,1
    (2, 3, 37, 35, 33, 7, 7, 2, 3),      # stem pattern
    (2, 3, 43, 47, 20, 11, 11, 4, 0),    # 16 phases
    (1, 5, 9, 10, 2, 1, 7, 1, 3),        # R != S
    (2, 17, 12, 12, 9, 1, 1, 1, 0),      # 1x1: no transform at all
    (1, 4, 16, 16, 8, 2, 2, 2, 0),
    (1, 3, 20, 18, 5, 4, 6, 3, 2),
    (5, 130, 7, 7, 129, 3, 3, 1, 1),     # long reduction, K and C off the tile sizes
    (2, 64, 30, 30, 64, 3, 3, 1, 1),     # several T tiles: whole tiles and split ones
    (1, 3, 9, 300, 4, 3, 5, 1, 2),       # one long row
    (4, 128, 28, 28, 96, 3, 3, 2, 1),    # the downsampling layer at a reduced size
]


@pytest.mark.parametrize("shape", SHAPES)
def test_f32out_matches_half_oracle(shape):
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand16(*shape, seed=500 + R * 7 + S + C)
    ref = oracle.dwm_bf16_f64(x, w, s, P)
    r = Bf16Runner(*shape)
    try:
        y = r.run(x, w, f32out=True)
    finally:
        r.close()
    assert np.all(np.isfinite(y))
    err = float(np.max(np.abs(y.astype(np.float64) - ref)) / np.max(np.abs(ref)))
    assert err <= TOL_F32OUT, err


@pytest.mark.parametrize("shape", SHAPES)
def test_half_out_within_one_step(shape):
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand16(*shape, seed=900 + R * 7 + S + C, dist="normal")
    ref = oracle.dwm_bf16_f64(x, w, s, P)
    r = Bf16Runner(*shape)
    try:
        y = r.run(x, w)
    finally:
        r.close()
    _check_half_out(y, ref)


@pytest.mark.parametrize("R,S,stride,pad", [(3, 3, 1, 1), (5, 5, 1, 2), (7, 7, 2, 3), (11, 11, 4, 0), (4, 6, 3, 2)])
def test_small_integers_are_exact(R, S, stride, pad):
    # every U and V is a small integer (w is a multiple of 4: G's halves stay integral), every
    # product and sum is exact in FP32: the result is the convolution itself
    rng = np.random.default_rng(R * 100 + S * 10 + stride)
    N, C, K, H = 2, 6, 37, max(R + 9, 18)
    x = rng.integers(-4, 5, size=(N, C, H, H + 1)).astype(np.float32)
    w = (4 * rng.integers(-3, 4, size=(K, C, R, S))).astype(np.float32)
    ref = oracle.direct_f64(x.astype(np.float32), w.astype(np.float32), stride, pad)
    r = Bf16Runner(N, C, H, H + 1, K, R, S, stride, pad)
    try:
        y = r.run(x, w, f32out=True)
    finally:
        r.close()
    assert np.array_equal(y.astype(np.float64), ref)


def test_rounding_points_closed_forms():
    # the cases that pin the oracle's rounding points (ties in U and in V), on the GPU
    h = 2.0 ** -8
    cases = [  # d (1x3 or 1x4 input), g (taps), expected y
        ([0.5, 1.0, 0.25], [1.0, h], [0.5, 1.0 + (0.25 - 1.0) * h]),
        ([0.0, 1.0, 1.0], [1.0, 3 * h], [-1.0 + (1.0 + 4 * h), None]),
        ([1.0, -h, 0.0], [1.0, 0.0], [1.0 - h, None]),
        ([0.0, -h, 1.0], [0.0, 1.0], [None, 1.0 - h]),
        ([0.0, 1.0, 0.0, 0.0], [1.0, h, 0.0], [0.5 - (0.5 - h / 2), 0.5 + (0.5 - h / 2)]),
    ]
    for d, g, want in cases:
        x = np.array(d, np.float32).reshape(1, 1, 1, len(d))
        w = np.array(g, np.float32).reshape(1, 1, 1, len(g))
        assert np.array_equal(x.astype(np.float64).reshape(-1), np.array(d))  # representable
        r = Bf16Runner(1, 1, 1, len(d), 1, 1, len(g), 1, 0)
        try:
            y = r.run(x, w, f32out=True).reshape(-1).astype(np.float64)
        finally:
            r.close()
        ref = oracle.dwm_bf16_f64(x, w, 1, 0).reshape(-1)
        assert np.array_equal(y, ref)
        for got, exp in zip(y, want):
            if exp is not None:
                assert got == exp


@pytest.mark.parametrize("variant", list(range(30, 48)))
def test_every_contraction_variant(variant):
    shape = (3, 64, 26, 26, 200, 3, 3, 1, 1)  # 64-row reductions: every chunk depth applies
    x, w = _rand16(*shape, seed=77)
    ref = oracle.dwm_bf16_f64(x, w, 1, 1)
    r = Bf16Runner(*shape, variant=variant)
    try:
        y = r.run(x, w, f32out=True)
        y16 = r.run(x, w)
    finally:
        r.close()
    err = float(np.max(np.abs(y.astype(np.float64) - ref)) / np.max(np.abs(ref)))
    assert err <= TOL_F32OUT, err
    _check_half_out(y16, ref)


@pytest.mark.parametrize("shape", [
    (3, 8, 19, 21, 70, 3, 3, 2, 1), (2, 24, 14, 14, 40, 7, 7, 1, 3), (2, 64, 30, 30, 64, 3, 3, 1, 1),
    (4, 128, 28, 28, 96, 3, 3, 2, 1), (1, 8, 11, 100, 20, 5, 5, 3, 1), (1, 40, 9, 130, 4, 3, 5, 1, 2),
    (70, 8, 6, 6, 8, 3, 3, 1, 1),  # blocks of 64 tiles that span several images
    (9, 8, 14, 14, 16, 7, 7, 2, 3),  # four images per block: a staged region beyond 64 KB
    (9, 16, 14, 14, 16, 11, 11, 2, 5),
    # channel counts that are not a multiple of eight: groups of eight rows across parts and channels
    (2, 3, 37, 35, 33, 7, 7, 2, 3), (2, 3, 43, 47, 20, 5, 5, 2, 2), (1, 5, 9, 10, 2, 1, 7, 1, 3),
    (3, 12, 20, 22, 24, 5, 5, 1, 2), (2, 20, 14, 14, 40, 3, 3, 1, 1), (70, 2, 6, 6, 3, 3, 3, 1, 1),
])
def test_input_transform_forms_agree(shape):
    """Gather form and LDS-staged form of the input transform produce the same V, hence the same
    output bits; both meet the bar."""
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand16(*shape, seed=1300 + R + C, dist="relu_normal")
    ref = oracle.dwm_bf16_f64(x, w, s, P)
    ys = []
    for form in (0, 1):
        r = Bf16Runner(*shape, input_variant=form)
        try:
            ys.append(r.run(x, w, f32out=True))
        finally:
            r.close()
    assert np.array_equal(ys[0].view(np.uint32), ys[1].view(np.uint32))
    err = float(np.max(np.abs(ys[1].astype(np.float64) - ref)) / np.max(np.abs(ref)))
    assert err <= TOL_F32OUT, err


def test_repeated_calls_give_identical_bits():
    shape = (2, 64, 30, 30, 64, 3, 3, 1, 1)
    x, w = _rand16(*shape, seed=3)
    r = Bf16Runner(*shape)
    try:
        a = r.run(x, w)
        b = r.run(x, w)
        c = r.run(x, w)
    finally:
        r.close()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(a.view(np.uint32), c.view(np.uint32))


@pytest.mark.parametrize("index", [1, 2])
def test_full_size_layers_sampled(index):
    """The benchmark layers at full size, in the launch configuration bench.py times: sampled
    outputs against the exact convolution of the bfloat16 inputs.  The half-precision result may
    be off by what bfloat16 storage of U, V and y costs: a few 2^-8 of the largest output."""
    L = wl.CONFIGS[index]
    x32, w32 = wl.make_layer_tensors(L, index)
    x, w = _bf(x32), _bf(w32)
    r = Bf16Runner(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    try:
        y = r.run(x, w)
    finally:
        r.close()
    assert np.all(np.isfinite(y))
    rng = np.random.default_rng(index)
    idx = rng.choice(y.size, size=4000, replace=False)
    ref = oracle.direct_f64_at(x.astype(np.float32), w.astype(np.float32), L.stride, L.pad, idx)
    got = y.reshape(-1)[idx].astype(np.float64)
    scale = float(np.max(np.abs(ref)))
    assert np.max(np.abs(got - ref)) <= 8 * 2.0 ** -8 * scale
    assert np.sqrt(np.mean((got - ref) ** 2)) <= 2 * 2.0 ** -8 * np.sqrt(np.mean(ref ** 2))


@pytest.mark.parametrize("index", [1, 2])
def test_full_size_layer_shapes_at_small_batch(index):
    """Same layer shapes, two images: element by element against the half oracle."""
    L = wl.CONFIGS[index]._replace(N=2)
    x32, w32 = wl.make_layer_tensors(L, index)
    x, w = _bf(x32), _bf(w32)
    ref = oracle.dwm_bf16_f64(x, w, L.stride, L.pad)
    r = Bf16Runner(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    try:
        y = r.run(x, w, f32out=True)
        y16 = r.run(x, w)
    finally:
        r.close()
    err = float(np.max(np.abs(y.astype(np.float64) - ref)) / np.max(np.abs(ref)))
    assert err <= TOL_F32OUT, err
    _check_half_out(y16, ref)


def test_error_codes():
    with pytest.raises(dwm.DwmError) as e:
        dwm.dwm_bf16_plan_create(1, 1, 2, 2, 1, 3, 3, 1, 0)  # kernel larger than the padded input
    assert e.value.status == dwm.DWM_ERR_INVALID_ARG
    plan = dwm.dwm_bf16_plan_create(1, 16, 8, 8, 4, 3, 3, 1, 1)
    dwm.dwm_bf16_set_variant(plan, "forward", 0)  # (the single kernel needs no workspace)
    try:
        buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_bf16_conv_forward(plan, buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), None)
        assert e.value.status == dwm.DWM_ERR_WORKSPACE
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_bf16_set_workspace(plan, buf.data_ptr(), 16)
        assert e.value.status == dwm.DWM_ERR_WORKSPACE
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_bf16_set_workspace(plan, buf.data_ptr() + 8, buf.numel() - 8)
        assert e.value.status == dwm.DWM_ERR_WORKSPACE
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_bf16_set_variant(plan, "contract", 12)  # a single-precision variant
        assert e.value.status == dwm.DWM_ERR_INVALID_ARG
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_bf16_set_variant(plan, "contract", 32)  # 64-row chunks on a 16-row layout
        assert e.value.status == dwm.DWM_ERR_INVALID_ARG
        p3 = dwm.dwm_bf16_plan_create(1, 70, 8, 8, 4, 3, 3, 1, 1)
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_bf16_set_variant(p3, "input", 1)  # the LDS-staged form needs C % 8 == 0 or C <= 64
        assert e.value.status == dwm.DWM_ERR_INVALID_ARG
        dwm.dwm_bf16_plan_destroy(p3)
    finally:
        dwm.dwm_bf16_plan_destroy(plan)


# ---- the single-kernel path (layers with few input channels) ----

def _single_kernel_applies(shape):
    p = dwm.dwm_bf16_plan_create(*shape)
    try:
        dwm.dwm_bf16_set_variant(p, "forward", 1)
        return True
    except dwm.DwmError:
        return False
    finally:
        dwm.dwm_bf16_plan_destroy(p)


SINGLE_SHAPES = [sh for sh in SHAPES if _single_kernel_applies(sh)] + [
    (3, 3, 64, 64, 64, 7, 7, 2, 3),      # the 7x7 stride-2 stem: classes (3,3), (3,1), (1,3), (1,1); one pass of four filter blocks
    (2, 3, 67, 67, 96, 11, 11, 4, 0),    # the 11x11 stride-4 stem: (3,3) with two steps, (3,2), (2,3), (2,2); two passes
    (2, 3, 50, 46, 13, 3, 3, 2, 1),      # K not a multiple of 16; classes (2,2), (2,1), (1,2), (1,1)
    (1, 1, 33, 35, 9, 5, 5, 2, 2),       # one channel
    (1, 7, 24, 24, 40, 5, 5, 1, 2),      # 3+2 taps, seven channels: steps that end inside a part
    (1, 12, 20, 22, 100, 3, 3, 1, 1),    # seven filter blocks: two passes, the second with three
    (2, 3, 9, 200, 6, 7, 7, 2, 3),       # a wide, flat image
    (600, 3, 30, 30, 5, 5, 5, 2, 2),     # more blocks than persistent workgroups
    (2, 20, 21, 19, 24, 3, 3, 1, 1),     # twenty channels: above the planner's own limit, forced
]


@pytest.mark.parametrize("shape", SINGLE_SHAPES)
def test_single_kernel_f32out_matches_oracle(shape):
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand16(*shape, seed=1500 + R * 7 + S + C)
    ref = oracle.dwm_bf16_f64(x, w, s, P)
    r = Bf16Runner(*shape, forward=1)
    try:
        assert r.info.forward_path == 1
        y = r.run(x, w, f32out=True)
    finally:
        r.close()
    assert np.all(np.isfinite(y))
    err = float(np.max(np.abs(y.astype(np.float64) - ref)) / np.max(np.abs(ref)))
    assert err <= TOL_F32OUT, err


@pytest.mark.parametrize("shape", SINGLE_SHAPES)
def test_single_kernel_16bit_out_within_one_step(shape):
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand16(*shape, seed=1900 + R * 7 + S + C, dist="normal")
    ref = oracle.dwm_bf16_f64(x, w, s, P)
    r = Bf16Runner(*shape, forward=1)
    try:
        y = r.run(x, w)
    finally:
        r.close()
    _check_half_out(y, ref)


@pytest.mark.parametrize("R,S,stride,pad", [(3, 3, 1, 1), (5, 5, 1, 2), (7, 7, 2, 3), (11, 11, 4, 0), (4, 6, 3, 2)])
def test_single_kernel_small_integers_are_exact(R, S, stride, pad):
    rng = np.random.default_rng(R * 100 + S * 10 + stride + 1)
    N, C, K, H = 2, 6, 37, max(R + 9, 18)
    x = rng.integers(-4, 5, size=(N, C, H, H + 1)).astype(np.float32)
    w = (4 * rng.integers(-3, 4, size=(K, C, R, S))).astype(np.float32)
    ref = oracle.direct_f64(x.astype(np.float32), w.astype(np.float32), stride, pad)
    r = Bf16Runner(N, C, H, H + 1, K, R, S, stride, pad, forward=1)
    try:
        y = r.run(x, w, f32out=True)
    finally:
        r.close()
    assert np.array_equal(y.astype(np.float64), ref)


@pytest.mark.parametrize("forward", [0, 1])
def test_input_transform_is_evaluated_in_binary32_before_its_rounding(forward):
    """The closed-form case that separates "V rounded from its binary32 evaluation" from "V rounded from its
    exact value" (derived at the oracle's test of the same name): both forward forms give the former."""
    a, b, c = 1 + 2.0 ** -6, 2.0 ** -8, 2.0 ** -24
    x = np.zeros((1, 1, 4, 4), np.float32)
    x[0, 0, 0, 0], x[0, 0, 2, 0], x[0, 0, 0, 2] = a, b, c
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 0, 0] = 1.0
    r = Bf16Runner(1, 1, 4, 4, 1, 3, 3, 1, 0, forward=forward)
    try:
        y = r.run(x, w, f32out=True).astype(np.float64)
    finally:
        r.close()
    ref = oracle.dwm_bf16_f64(x, w, 1, 0)
    assert ref[0, 0, 0, 0] == (1 + 2.0 ** -6) + c + b
    assert abs(y[0, 0, 0, 0] - ref[0, 0, 0, 0]) <= 2.0 ** -23  # (FP32 accumulation of the 2^-24 beside 1)
    assert np.max(np.abs(y - ref)) <= 2.0 ** -23


def test_single_kernel_rounding_points():
    """The cases that pin the oracle's rounding points: one product per output, so the single kernel
    must reproduce the oracle bit for bit."""
    h = 2.0 ** -8
    cases = [([0.5, 1.0, 0.25], [1.0, h]), ([0.0, 1.0, 1.0], [1.0, 3 * h]), ([1.0, -h, 0.0], [1.0, 0.0]),
             ([0.0, -h, 1.0], [0.0, 1.0]), ([0.0, 1.0, 0.0, 0.0], [1.0, h, 0.0])]
    for d, g in cases:
        x = np.array(d, np.float32).reshape(1, 1, 1, len(d))
        w = np.array(g, np.float32).reshape(1, 1, 1, len(g))
        r = Bf16Runner(1, 1, 1, len(d), 1, 1, len(g), 1, 0, forward=1)
        try:
            y = r.run(x, w, f32out=True).reshape(-1).astype(np.float64)
        finally:
            r.close()
        assert np.array_equal(y, oracle.dwm_bf16_f64(x, w, 1, 0).reshape(-1))


@pytest.mark.parametrize("index", [3, 4])
def test_stems_full_size_planner_choice(index):
    """The two stems at full size with the planner's own choice of path (the single kernel): sampled
    outputs against the exact convolution of the 16-bit inputs, and two images element by element
    against the oracle."""
    L = wl.CONFIGS[index]
    x32, w32 = wl.make_layer_tensors(L, index)
    x, w = _bf(x32), _bf(w32)
    r = Bf16Runner(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, forward=-1)
    try:
        assert r.info.forward_path == 1
        y = r.run(x, w)
        y32 = r.run(x, w, f32out=True)
    finally:
        r.close()
    assert np.all(np.isfinite(y))
    rng = np.random.default_rng(index)
    idx = rng.choice(y.size, size=4000, replace=False)
    ref = oracle.direct_f64_at(np.asarray(x, np.float32), np.asarray(w, np.float32), L.stride, L.pad, idx)
    got = y.reshape(-1)[idx].astype(np.float64)
    scale = float(np.max(np.abs(ref)))
    assert np.max(np.abs(got - ref)) <= 8 * 2.0 ** -8 * scale
    ref2 = oracle.dwm_bf16_f64(x[:2], w, L.stride, L.pad)
    err = float(np.max(np.abs(y32[:2].astype(np.float64) - ref2)) / np.max(np.abs(ref2)))
    assert err <= TOL_F32OUT, err
    _check_half_out(y[:2], ref2)


def test_single_kernel_refused_where_it_does_not_apply():
    p = dwm.dwm_bf16_plan_create(1, 200, 8, 8, 4, 3, 3, 1, 1)  # 200 channels
    try:
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_bf16_set_variant(p, "forward", 1)
        assert e.value.status == dwm.DWM_ERR_INVALID_ARG
        assert dwm.dwm_bf16_plan_info(p).forward_path == 0
    finally:
        dwm.dwm_bf16_plan_destroy(p)


@pytest.mark.parametrize("shape", [
    (3, 3, 64, 64, 64, 7, 7, 2, 3),      # classes (3,3), (3,1), (1,3), (1,1)
    (2, 3, 67, 67, 96, 11, 11, 4, 0),    # (3,3), (3,2), (2,3), (2,2)
    (2, 3, 50, 46, 13, 3, 3, 2, 1),      # (2,2), (2,1), (1,2), (1,1)
    (1, 12, 20, 22, 100, 3, 3, 1, 1),    # (3,3) alone
    (1, 7, 24, 24, 40, 5, 5, 1, 2),      # (3,3), (3,2), (2,3), (2,2) with steps that end inside a part
])
def test_single_kernel_general_and_built_for_the_classes_agree(shape):
    """The kernel built for the layer's list of classes (four filter blocks per pass) and the general
    one (class switch, two blocks per pass) issue the same MFMAs in the same order per output: the
    same bits; the general one is then also checked against the oracle."""
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand16(*shape, seed=2300 + R + C, dist="relu_normal")
    ys = []
    for classes in (-1, 0):
        r = Bf16Runner(*shape, forward=1, classes=classes)
        try:
            ys.append(r.run(x, w, f32out=True))
        finally:
            r.close()
    assert np.array_equal(ys[0].view(np.uint32), ys[1].view(np.uint32))
    ref = oracle.dwm_bf16_f64(x, w, s, P)
    err = float(np.max(np.abs(ys[1].astype(np.float64) - ref)) / np.max(np.abs(ref)))
    assert err <= TOL_F32OUT, err
