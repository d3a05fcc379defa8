"""GPU parity tests of the data gradient: dwm_conv_backward_data, called through the C ABI,
against the FP64 definition of dL/dx (oracle.backward_data_f64).

Bar: max |dx_gpu - dx_ref| / max |dx_ref| <= 1e-4, the forward path's bar (the gradient is a
sum of K*R*S/stride^2 products per pixel in the same fp32 arithmetic).
"""
import numpy as np
import pytest
import torch

import dwm_workloads as wl
import oracle
import paper_2002_00552_amd as dwm

pytestmark = pytest.mark.gpu

TOL = 1e-4


class BwdRunner:
    def __init__(self, N, C, H, W, K, R, S, stride, pad, path=-1):
        self.plan = dwm.dwm_bwd_data_plan_create(N, C, H, W, K, R, S, stride, pad)
        dwm.dwm_bwd_data_set_variant(self.plan, "path", path)
        dev = torch.device("cuda:0")
        self.Ugw = torch.full((dwm.dwm_bwd_data_filter_bytes(self.plan) // 4,), float("nan"), dtype=torch.float32, device=dev)
        self.ws = torch.full((max(dwm.dwm_bwd_data_workspace_bytes(self.plan) // 4, 64),), float("nan"),
                             dtype=torch.float32, device=dev)
        dwm.dwm_bwd_data_set_workspace(self.plan, self.ws.data_ptr(), self.ws.numel() * 4)
        self.dx = torch.full((N, C, H, W), float("nan"), dtype=torch.float32, device=dev)

    def run(self, dy, w):
        st = torch.cuda.current_stream().cuda_stream
        self.w = torch.from_numpy(np.ascontiguousarray(w)).cuda()
        self.dy = torch.from_numpy(np.ascontiguousarray(dy)).cuda()
        dwm.dwm_bwd_data_filter_transform(self.plan, self.w.data_ptr(), self.Ugw.data_ptr(), st)
        dwm.dwm_conv_backward_data(self.plan, self.dy.data_ptr(), self.Ugw.data_ptr(), self.dx.data_ptr(), st)
        torch.cuda.synchronize()
        return self.dx.cpu().numpy()

    def close(self):
        dwm.dwm_bwd_data_plan_destroy(self.plan)


def _rand(N, C, H, W, K, R, S, s, P, seed):
    rng = np.random.default_rng(seed)
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    w = (rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)
    dy = rng.uniform(-1, 1, (N, K, OH, OW)).astype(np.float32)
    return w, dy


def _relerr(a, ref):
    return float(np.max(np.abs(a.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


SHAPES = [  # N, C, H, W, K, R, S, stride, pad
    (1, 16, 32, 32, 16, 5, 5, 1, 2),     # benchmark config 1
    (2, 3, 13, 15, 5, 5, 5, 1, 2),
    (3, 8, 19, 21, 70, 3, 3, 2, 1),      # the stride-2 downsampling pattern, odd sizes
    (2, 24, 14, 14, 40, 7, 7, 1, 3),
    (2, 3, 37, 35, 33, 7, 7, 2, 3),      # stem pattern: phases of 4 and 3 taps
    (2, 3, 43, 47, 20, 11, 11, 4, 0),    # 16 phases, pixels at the end no window touches
    (1, 5, 9, 10, 2, 1, 7, 1, 3),        # R != S
    (2, 17, 12, 12, 9, 1, 1, 1, 0),      # 1x1
    (1, 7, 11, 11, 4, 1, 1, 2, 0),       # stride beyond the kernel: three of four phases are zeros
    (1, 4, 16, 16, 8, 2, 2, 2, 0),
    (1, 3, 20, 18, 5, 4, 6, 3, 2),       # pad not a multiple of the stride
    (1, 2, 12, 12, 3, 12, 12, 1, 0),     # a single output pixel spread over the whole image
    (5, 130, 7, 7, 129, 3, 3, 1, 1),     # many channels on both sides: staged sub-convolutions
    (2, 70, 21, 19, 130, 3, 3, 2, 1),
    (1, 3, 9, 300, 4, 3, 5, 1, 2),       # one long row
    (2, 6, 40, 33, 5, 5, 5, 2, 5),       # pad larger than the kernel reach: windows wholly in the padding
    (1, 5, 20, 18, 140, 4, 6, 3, 2),     # nine sub-convolutions of different extents contracted in one launch
    (2, 9, 17, 22, 200, 5, 5, 2, 2),     # four, 3- and 2-tap phases: several classes per sub-convolution
    (1, 4, 23, 23, 130, 11, 11, 4, 0),   # sixteen: too many planes for one table, run one after the other
    (2, 10, 20, 24, 150, 3, 3, 2, 1),    # even sizes: equal tile grids, ONE input transform for the four sub-convolutions
    (1, 6, 16, 16, 130, 7, 7, 2, 3),     # the same with nine classes in the merged plan (3+1 and 3 taps per phase)
    (1, 4, 18, 18, 140, 5, 5, 3, 1),     # stride 3: nine sub-convolutions of 2x2 .. 1x1 taps
    (3, 5, 12, 12, 128, 2, 2, 2, 0),     # one tap per phase: four 1x1 sub-convolutions
]


def _single_kernel_applies(shape):
    """Host-side question to the plan: can the whole gradient run as one kernel?"""
    p = dwm.dwm_bwd_data_plan_create(*shape)
    try:
        dwm.dwm_bwd_data_set_variant(p, "path", 1)
        return True
    except dwm.DwmError:
        return False
    finally:
        dwm.dwm_bwd_data_plan_destroy(p)


SMALL_SHAPES = [sh for sh in SHAPES if _single_kernel_applies(sh)] + [
    # stems: few input channels, many filters, the window of dy cut 2+2 / 3 / 3+2
    (3, 3, 64, 64, 64, 7, 7, 2, 3),      # 4x4 window, nine planes, 12 columns, several chunks of channels
    (2, 3, 67, 67, 96, 11, 11, 4, 0),    # 3x3 window, sixteen planes, three blocks of 16 columns, odd image
    (2, 3, 67, 67, 20, 11, 11, 4, 2),    # padding shifts the residues: a 4-tap window for an 11-tap kernel
    (2, 3, 50, 46, 13, 3, 3, 2, 1),      # 2x2 window: one pair of pieces, K not a multiple of the chunk
    (1, 1, 33, 35, 9, 5, 5, 2, 2),       # one channel: 4 of 16 columns in use
    (2, 4, 30, 30, 10, 9, 9, 3, 4),      # stride 3: the general scatter of the columns
    (1, 3, 40, 40, 7, 6, 6, 1, 2),       # stride 1, six taps: 3+3
    (1, 2, 26, 30, 5, 10, 10, 2, 3),     # ten taps, stride 2: a window of six
    (2, 3, 45, 41, 11, 9, 9, 2, 4),      # nine taps, stride 2: a window of five, 3+2
    (1, 8, 24, 24, 12, 6, 6, 2, 2),      # 32 columns
    (2, 3, 9, 200, 6, 7, 7, 2, 3),       # a wide, flat image: blocks of one row of tiles
    (600, 3, 12, 12, 5, 5, 5, 2, 2),     # more blocks than persistent workgroups: each takes several
    (1, 16, 20, 20, 6, 4, 4, 2, 1),      # 64 columns: two groups of two column blocks per wave
    (1, 5, 18, 22, 7, 7, 7, 4, 3),       # 80 columns: a group of three blocks, then two and a padding block
    (2, 7, 15, 17, 9, 5, 5, 3, 1),       # 63 columns, stride 3: the last block one column short
]


@pytest.mark.parametrize("shape", SHAPES)
def test_backward_data_matches_fp64_definition(shape):
    """The sub-convolution form (the planner's choice where the layer has many channels)."""
    N, C, H, W, K, R, S, s, P = shape
    w, dy = _rand(*shape, seed=300 + R * 7 + S)
    ref = oracle.backward_data_f64(dy, w, (N, C, H, W), s, P)
    r = BwdRunner(*shape, path=0)
    dx = r.run(dy, w)
    r.close()
    assert np.all(np.isfinite(dx))  # every pixel written, the untouched ones as zeros
    assert _relerr(dx, ref) <= TOL, shape


@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_backward_data_single_kernel_matches_fp64_definition(shape):
    """The whole gradient as one stride-1 correlation of dy in one kernel."""
    N, C, H, W, K, R, S, s, P = shape
    w, dy = _rand(*shape, seed=900 + R * 7 + S)
    ref = oracle.backward_data_f64(dy, w, (N, C, H, W), s, P)
    r = BwdRunner(*shape, path=1)
    dx = r.run(dy, w)
    r.close()
    assert np.all(np.isfinite(dx))  # every pixel written, the untouched ones as zeros
    assert _relerr(dx, ref) <= TOL, shape


def test_backward_data_where_no_tap_reaches_the_image():
    """Stride above the kernel size on a one-pixel-wide image: every pixel of dx is untouched by the forward
    pass, the plan has no sub-convolution and no transformed filter (zero bytes: no buffer is passed), dx = 0."""
    shape = (7, 7, 42, 1, 170, 2, 2, 3, 2)
    N, C, H, W, K, R, S, s, P = shape
    w, dy = _rand(*shape, seed=41)
    ref = oracle.backward_data_f64(dy, w, (N, C, H, W), s, P)
    assert not ref.any()
    plan = dwm.dwm_bwd_data_plan_create(*shape)
    try:
        assert dwm.dwm_bwd_data_filter_bytes(plan) == 0 and dwm.dwm_bwd_data_plan_info(plan).n_subconvs == 0
        st = torch.cuda.current_stream().cuda_stream
        wd, dyd = torch.from_numpy(w).cuda(), torch.from_numpy(dy).cuda()
        dx = torch.full((N, C, H, W), float("nan"), dtype=torch.float32, device="cuda:0")
        ws = torch.zeros(max(dwm.dwm_bwd_data_workspace_bytes(plan) // 4, 64), dtype=torch.float32, device="cuda:0")
        dwm.dwm_bwd_data_set_workspace(plan, ws.data_ptr(), ws.numel() * 4)
        dwm.dwm_bwd_data_filter_transform(plan, wd.data_ptr(), None, st)
        dwm.dwm_conv_backward_data(plan, dyd.data_ptr(), None, dx.data_ptr(), st)
        torch.cuda.synchronize()
        assert not dx.cpu().numpy().any()
    finally:
        dwm.dwm_bwd_data_plan_destroy(plan)


def test_backward_data_is_deterministic_and_plan_reusable():
    shape = (2, 8, 21, 20, 9, 5, 5, 2, 2)
    w, dy = _rand(*shape, seed=5)
    r = BwdRunner(*shape)
    a = r.run(dy, w).copy()
    r.dx.fill_(float("nan"))
    b = r.run(dy, w).copy()
    assert np.array_equal(a, b)
    dy2 = (dy * 0.5).astype(np.float32)
    c = r.run(dy2, w)
    assert _relerr(c, oracle.backward_data_f64(dy2, w, shape[:4], 2, 2)) <= TOL
    r.close()


def test_backward_data_phases_cover_the_image_once():
    for shape in [(1, 2, 17, 19, 3, 7, 7, 2, 3), (1, 2, 23, 22, 3, 11, 11, 4, 0), (1, 2, 9, 9, 3, 1, 1, 3, 0),
                  (1, 2, 10, 13, 3, 4, 6, 3, 2)]:
        N, C, H, W, K, R, S, s, P = shape
        p = dwm.dwm_bwd_data_plan_create(*shape)
        info = dwm.dwm_bwd_data_plan_info(p)
        assert info.n_phases == s * s
        cover = np.zeros((H, W), int)
        for i in range(info.n_phases):
            ph = dwm.dwm_bwd_data_plan_phase(p, i)
            assert ph.taps_h == len(range(ph.phase_h, R, s)) and ph.taps_w == len(range(ph.phase_w, S, s))
            if ph.count_h > 0 and ph.count_w > 0:
                cover[ph.first_h:ph.first_h + s * ph.count_h:s, ph.first_w:ph.first_w + s * ph.count_w:s] += 1
                assert (ph.first_h + P) % s == ph.phase_h and (ph.first_w + P) % s == ph.phase_w
                assert bool(ph.has_subconv) == (ph.taps_h > 0 and ph.taps_w > 0)
        assert np.all(cover == 1)
        dwm.dwm_bwd_data_plan_destroy(p)


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_backward_data_benchmark_layers_full_size(index):
    """Whole layer on the GPU, EVERY pixel of dx compared with the FP64 definition."""
    L = wl.CONFIGS[index]
    _, w = wl.make_layer_tensors(L, index)
    OH, OW = wl.out_hw(L)
    dy = np.random.default_rng(3100 + index).uniform(-1, 1, (L.N, L.K, OH, OW)).astype(np.float32)
    print("data gradient, whole image:", L.name, flush=True)
    r = BwdRunner(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)  # the planner's choice of path
    dx = r.run(dy, w)
    r.close()
    assert dx.shape == (L.N, L.C, L.H, L.W) and np.all(np.isfinite(dx))
    ref = oracle.backward_data_f64(dy, w, (L.N, L.C, L.H, L.W), L.stride, L.pad)
    err = np.abs(dx - ref)
    worst = np.unravel_index(np.argmax(err), err.shape)
    assert err[worst] / np.max(np.abs(ref)) <= TOL, (L.name, worst)


# ---- gradient with respect to the filter ----

class WgradRunner:
    def __init__(self, N, C, H, W, K, R, S, stride, pad):
        self.plan = dwm.dwm_bwd_filter_plan_create(N, C, H, W, K, R, S, stride, pad)
        dev = torch.device("cuda:0")
        self.ws = torch.full((dwm.dwm_bwd_filter_workspace_bytes(self.plan) // 4,), float("nan"),
                             dtype=torch.float32, device=dev)
        dwm.dwm_bwd_filter_set_workspace(self.plan, self.ws.data_ptr(), self.ws.numel() * 4)
        self.dw = torch.full((K, C, R, S), float("nan"), dtype=torch.float32, device=dev)

    def run(self, x, dy):
        st = torch.cuda.current_stream().cuda_stream
        self.x = torch.from_numpy(np.ascontiguousarray(x)).cuda()
        self.dy = torch.from_numpy(np.ascontiguousarray(dy)).cuda()
        dwm.dwm_conv_backward_filter(self.plan, self.x.data_ptr(), self.dy.data_ptr(), self.dw.data_ptr(), st)
        torch.cuda.synchronize()
        return self.dw.cpu().numpy()

    def close(self):
        dwm.dwm_bwd_filter_plan_destroy(self.plan)


def _rand_xdy(N, C, H, W, K, R, S, s, P, seed):
    rng = np.random.default_rng(seed)
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    dy = rng.uniform(-1, 1, (N, K, OH, OW)).astype(np.float32)
    return x, dy


WSHAPES = SHAPES + [
    (70, 2, 6, 6, 3, 3, 3, 1, 1),        # many images: the tile axis spans several blocks and ranges
    (3, 5, 31, 33, 7, 5, 5, 1, 2),       # tile count not a multiple of 64: the zeroed tail columns
    (2, 66, 12, 12, 67, 3, 3, 1, 1),     # channels and filters just past a 64 tile
    # few channels and many tiles: the short-reduction form (dy straight into the MFMA)
    (8, 3, 190, 181, 20, 7, 7, 2, 3),    # odd output sizes: masked rows and columns of dy, tail of the tile axis
    (21, 3, 227, 227, 33, 11, 11, 4, 0), # a class with two blocks of sixteen rows
    (4, 4, 128, 130, 70, 5, 5, 1, 2),    # filters past one 64-filter tile
    (16, 6, 130, 127, 16, 3, 3, 2, 1),   # classes of 2-tap and 1-tap pieces
    (9, 3, 180, 180, 20, 9, 9, 2, 4),    # phases of five and four taps: sixteen parts in four classes, one launch
]


@pytest.mark.parametrize("shape", WSHAPES)
def test_backward_filter_matches_fp64_definition(shape):
    N, C, H, W, K, R, S, s, P = shape
    x, dy = _rand_xdy(*shape, seed=700 + R * 7 + S)
    ref = oracle.backward_filter_f64(x, dy, (K, C, R, S), s, P)
    r = WgradRunner(*shape)
    dw = r.run(x, dy)
    r.close()
    assert np.all(np.isfinite(dw))  # every tap written
    assert _relerr(dw, ref) <= TOL, shape


def test_backward_filter_is_deterministic_and_plan_reusable():
    shape = (4, 8, 21, 20, 9, 5, 5, 2, 2)
    x, dy = _rand_xdy(*shape, seed=6)
    r = WgradRunner(*shape)
    a = r.run(x, dy).copy()
    r.dw.fill_(float("nan"))
    b = r.run(x, dy).copy()
    assert np.array_equal(a, b)
    x2 = (x * 0.5).astype(np.float32)
    c = r.run(x2, dy)
    assert _relerr(c, oracle.backward_filter_f64(x2, dy, (9, 8, 5, 5), 2, 2)) <= TOL
    r.close()


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_backward_filter_benchmark_layers_full_size(index):
    """Whole layer on the GPU, EVERY tap of every filter compared with the FP64 definition."""
    L = wl.CONFIGS[index]
    x, _ = wl.make_layer_tensors(L, index)
    OH, OW = wl.out_hw(L)
    dy = np.random.default_rng(4100 + index).uniform(-1, 1, (L.N, L.K, OH, OW)).astype(np.float32)
    print("filter gradient, all filters:", L.name, flush=True)
    r = WgradRunner(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    dw = r.run(x, dy)
    r.close()
    assert dw.shape == (L.K, L.C, L.R, L.S) and np.all(np.isfinite(dw))
    ref = oracle.backward_filter_f64(x, dy, (L.K, L.C, L.R, L.S), L.stride, L.pad)
    err = np.abs(dw - ref)
    worst = np.unravel_index(np.argmax(err), err.shape)
    assert err[worst] / np.max(np.abs(ref)) <= TOL, (L.name, worst)
