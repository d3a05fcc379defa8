"""GPU parity tests: the HIP path, called through the C ABI, against the FP64 oracle.

Bar (stated by the task's target): max |y_gpu - y_ref| / max |y_ref| <= 1e-4 with y_ref the
FP64 direct convolution of the same float32 inputs.  Stage outputs (U, V) are exact up to
fp32 rounding of a handful of additions, so they get 1e-6 relative to their max.
"""
import numpy as np
import pytest
import torch

import dwm_workloads as wl
import oracle
import paper_2002_00552_amd as dwm
from dwm_gpu import Runner, conv

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _rand(N, C, H, W, K, R, S, seed):
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)
    return x, w


def _relerr(y, ref):
    return float(np.max(np.abs(y.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def _part_tuple(pt):
    return (pt.phase_h, pt.off_h, pt.len_h, pt.phase_w, pt.off_w, pt.len_w)


# ---- stage parity: filter transform and input transform against the oracle's stages ----

STAGE_SHAPES = [  # N, C, H, W, K, R, S, stride, pad
    (2, 3, 13, 15, 5, 5, 5, 1, 2),
    (1, 4, 17, 12, 6, 3, 3, 2, 1),
    (2, 3, 23, 22, 4, 7, 7, 2, 3),
    (1, 2, 31, 29, 3, 11, 11, 4, 0),
    (1, 5, 9, 10, 2, 1, 7, 1, 3),
    (1, 20, 8, 8, 130, 3, 3, 1, 1),
    (1, 2, 150, 700, 2, 5, 5, 2, 2),     # wide image: several bands of tile rows
    (1, 1, 90, 500, 1, 11, 11, 4, 0),
]


@pytest.mark.parametrize("shape", STAGE_SHAPES)
def test_filter_transform_matches_oracle(shape):
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand(*shape[:7], seed=11)
    r = Runner(*shape)
    r.Ugw.fill_(float("nan"))
    r.set_filter(w)
    torch.cuda.synchronize()
    U = r.Ugw.cpu().numpy()
    assert np.all(np.isfinite(U))  # padding included: it must be written (as zeros)
    classes, Kpad = r.classes(), r.info.Kpad
    seen = np.zeros(U.size, bool)
    for pt in r.parts():
        q = classes[pt.cls]
        th, tw = q.len_h + 1, q.len_w + 1
        Ug = U[q.u_offset:q.u_offset + th * tw * Kpad * q.Lpad].reshape(th, tw, Kpad, q.Lpad)
        ref = oracle.part_filter_transform(w, s, _part_tuple(pt))  # [K][C][th][tw]
        got = Ug[:, :, :K, pt.slot * C:(pt.slot + 1) * C].transpose(2, 3, 0, 1)
        assert np.max(np.abs(got - ref)) <= 1e-6 * max(np.max(np.abs(ref)), 1e-30)
        # padding rows/columns are zero
        assert np.all(Ug[:, :, K:, :] == 0) and np.all(Ug[:, :, :, q.L:] == 0)
    # the single-kernel path's copy: (part, channel) rows with the F(2,2) form that shares the
    # frequencies of F(2,3) (the oracle's form 1)
    nfc, nrows, nslices = dwm.dwm_plan_fused_info(r.plan)
    if nfc:
        oracle.set_f22_form(1)
        try:
            parts = r.parts()
            refs = [oracle.part_filter_transform(w, s, _part_tuple(pt)) for pt in parts]  # [K][C][th][tw]
        finally:
            oracle.set_f22_form(0)
        scale = max(np.max(np.abs(u)) for u in refs)
        for i in range(nfc):
            fq = dwm.dwm_plan_fused_class(r.plan, i)
            n = nslices * fq.n_freq_h * fq.n_freq_w * fq.rows * 32
            UF = U[fq.uf_offset:fq.uf_offset + n].reshape(nslices, fq.n_freq_h, fq.n_freq_w, fq.rows, 16, 2)
            # filter index = 32*slice + 16*half + i  ->  [fh][fw][row][filter]
            UF = UF.transpose(1, 2, 3, 0, 5, 4).reshape(fq.n_freq_h, fq.n_freq_w, fq.rows, nslices * 32)
            assert np.all(UF[:, :, :, K:] == 0)
            for j in range(fq.rows):
                row = dwm.dwm_plan_fused_row(r.plan, fq.first_row + j)
                pt = parts[row.part]
                want = np.zeros((fq.n_freq_h, fq.n_freq_w, K))
                if row.real:
                    want[:pt.len_h + 1, :pt.len_w + 1, :] = refs[row.part][:, row.channel].transpose(1, 2, 0)
                assert np.max(np.abs(UF[:, :, j, :K] - want)) <= 1e-6 * scale, (i, j)
    r.close()


@pytest.mark.parametrize("shape", STAGE_SHAPES)
def test_input_transform_matches_oracle(shape):
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand(*shape[:7], seed=12)
    r = Runner(*shape)
    xd = torch.from_numpy(x).cuda()
    dwm.dwm_input_transform(r.plan, xd.data_ptr(), r.stream())
    torch.cuda.synchronize()
    info, classes = r.info, r.classes()
    TH, TW, T, Tpad = info.TH, info.TW, info.T, info.Tpad
    # V is blocked by 64 tiles: [block][row][64] -> [row][t]
    rows = info.Vblock // 64
    V = r.ws.cpu().numpy()[:(Tpad // 64) * info.Vblock].reshape(Tpad // 64, rows, 64)
    V = V.transpose(1, 0, 2).reshape(rows, Tpad)
    for pt in r.parts():
        q = classes[pt.cls]
        th, tw = q.len_h + 1, q.len_w + 1
        row0 = q.v_offset // 64
        Vg = V[row0:row0 + th * tw * q.Lpad].reshape(th, tw, q.Lpad, Tpad)
        assert np.all(Vg[:, :, q.L:, :T] == 0)  # padded reduction rows must be zero
        for n in range(N):
            ref = oracle.part_input_transform(x, R, S, s, P, _part_tuple(pt), n)  # [C][TH][TW][th][tw]
            got = Vg[:, :, pt.slot * C:(pt.slot + 1) * C, n * TH * TW:(n + 1) * TH * TW]
            got = got.reshape(th, tw, C, TH, TW).transpose(2, 3, 4, 0, 1)
            assert np.max(np.abs(got - ref)) <= 1e-6 * max(np.max(np.abs(ref)), 1e-30), (_part_tuple(pt), n)
    r.close()


def _v_rows(r):
    """The transformed input as [row][t], t < T, from the plan's workspace (blocked by 64 tiles)."""
    info = r.info
    rows = info.Vblock // 64
    V = r.ws.cpu().numpy()[:(info.Tpad // 64) * info.Vblock].reshape(info.Tpad // 64, rows, 64)
    return V.transpose(1, 0, 2).reshape(rows, info.Tpad)[:, :info.T]


FORM_SHAPES = [
    (2, 3, 23, 22, 4, 7, 7, 2, 3),
    (3, 9, 14, 14, 5, 7, 7, 1, 3),       # a block of 64 tiles spans three images
    (70, 5, 6, 6, 3, 3, 3, 1, 1),        # ... and here eight
    (1, 6, 31, 29, 3, 11, 11, 4, 0),
    (2, 10, 19, 21, 7, 3, 3, 2, 1),
    (1, 4, 9, 300, 4, 3, 5, 1, 2),       # rows wider than one wave
    (1, 2, 150, 700, 3, 5, 5, 2, 2),
    (2, 7, 12, 12, 9, 1, 1, 2, 0),       # kernel shorter than the stride
]


@pytest.mark.parametrize("shape", FORM_SHAPES)
def test_input_transform_forms_agree(shape):
    """The gather form (variants 0, 1) and the LDS-staged form (2, 3; any channel group size)
    apply the same additions in the same order: V must be bit-identical."""
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand(*shape[:7], seed=21)
    xd = torch.from_numpy(x).cuda()
    ref = None
    for variant, cg in [(0, 0), (1, 0), (2, 0), (3, 0), (2, 1), (2, min(C, 3)), (3, min(C, 8))]:
        r = Runner(*shape)
        if cg:
            dwm.dwm_plan_set_variant(r.plan, "input_cg", cg)
        dwm.dwm_plan_set_variant(r.plan, "input", variant)
        dwm.dwm_input_transform(r.plan, xd.data_ptr(), r.stream())
        torch.cuda.synchronize()
        V = _v_rows(r).copy()
        r.close()
        assert np.all(np.isfinite(V)), (variant, cg)
        if ref is None:
            ref = V
        else:
            assert np.array_equal(V, ref), (variant, cg)


def test_input_transform_falls_back_when_rows_do_not_fit_in_lds():
    """A very wide image: the staged rows of one block exceed LDS, so only the gather form
    applies; the planner must choose it and refuse the other."""
    shape = (1, 2, 12, 6000, 3, 3, 3, 1, 1)
    x, w = _rand(*shape[:7], seed=22)
    ref = oracle.direct_f64(x, w, 1, 1)
    p = dwm.dwm_plan_create(*shape)
    with pytest.raises(dwm.DwmError):
        dwm.dwm_plan_set_variant(p, "input", 2)
    dwm.dwm_plan_destroy(p)
    y = conv(x, w, 1, 1, variants={"forward": 0})
    assert _relerr(y, ref) <= TOL


# ---- end-to-end parity on small shapes that span several tiles and ragged tails ----

E2E_SHAPES = [
    (1, 16, 32, 32, 16, 5, 5, 1, 2),     # benchmark config 1
    (2, 3, 13, 15, 5, 5, 5, 1, 2),
    (3, 8, 19, 21, 70, 3, 3, 2, 1),      # K crosses a 64 tile, odd output
    (2, 24, 14, 14, 40, 7, 7, 1, 3),
    (2, 3, 37, 35, 33, 7, 7, 2, 3),
    (2, 3, 43, 47, 20, 11, 11, 4, 0),    # odd OH/OW, 16 phases
    (1, 5, 9, 10, 2, 1, 7, 1, 3),        # R != S
    (1, 6, 10, 9, 3, 7, 1, 1, 3),
    (2, 17, 12, 12, 9, 1, 1, 1, 0),      # 1x1: a single one-tap part
    (1, 7, 11, 11, 4, 1, 1, 2, 0),       # stride beyond the kernel
    (1, 4, 16, 16, 8, 2, 2, 2, 0),
    (1, 3, 20, 18, 5, 4, 6, 3, 2),       # pad not a multiple of the stride
    (1, 2, 12, 12, 3, 12, 12, 1, 0),     # a single output pixel
    (5, 130, 7, 7, 129, 3, 3, 1, 1),     # reduction and K just past tile boundaries
    (70, 2, 6, 6, 3, 3, 3, 1, 1),        # many images, T crosses several T tiles
    (1, 3, 9, 300, 4, 3, 5, 1, 2),       # one long row
    (1, 2, 150, 700, 3, 5, 5, 2, 2),     # several bands of tile rows in the input transform
    (2, 2, 301, 64, 3, 7, 3, 1, 3),      # tall image
    (3, 16, 56, 56, 256, 5, 5, 1, 2),    # 148 long tiles on 256 CUs: every tile is cut into two ranges of its own
    (11, 32, 56, 56, 256, 5, 5, 2, 2),   # the same with 136 tiles of 49 32-step chunks (odd: ranges of 25 and 24)
    (6, 12, 68, 10, 116, 10, 10, 4, 3),  # one tile per row: a block of 64 tiles stages whole images, 45 KB a channel
]


@pytest.mark.parametrize("path", ["staged", "auto"])
@pytest.mark.parametrize("shape", E2E_SHAPES)
def test_forward_matches_fp64_direct(shape, path):
    """'staged' forces input transform + contraction; 'auto' lets the planner use the
    single-kernel path where it applies (few input channels)."""
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand(*shape[:7], seed=100 + R * 7 + S)
    ref = oracle.direct_f64(x, w, s, P)
    y = conv(x, w, s, P, variants={"forward": 0 if path == "staged" else -1})
    assert y.shape == ref.shape
    assert np.all(np.isfinite(y))
    assert _relerr(y, ref) <= TOL, shape


# every variant of the contraction kernel on shapes it applies to: chunks of 32 or 64 reduction steps need
# classes whose padded reduction length is a multiple of that (64 input channels here); 16-step chunks
# apply everywhere
_CHUNK16, _ALL = [10, 17], [10, 11, 12, 13, 14, 15, 16, 17, 18, 19]
VARIANT_CASES = [(shape, v) for shape, vs in [
    ((3, 8, 19, 21, 70, 3, 3, 2, 1), _CHUNK16),
    ((2, 24, 30, 30, 140, 7, 7, 1, 3), _CHUNK16),
    ((2, 3, 43, 47, 20, 11, 11, 4, 0), _CHUNK16),
    ((3, 64, 19, 21, 70, 3, 3, 2, 1), _ALL),
    ((2, 64, 14, 18, 130, 5, 5, 1, 2), _ALL),
    ((5, 128, 30, 30, 150, 3, 3, 1, 1), _ALL),   # 30 tiles of 64x64: every tile cut into ranges, partial sums
] for v in vs]


@pytest.mark.parametrize("shape,variant", VARIANT_CASES)
def test_every_contraction_variant(shape, variant):
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand(*shape[:7], seed=5)
    ref = oracle.direct_f64(x, w, s, P)
    y = conv(x, w, s, P, variants={"contract": variant, "forward": 0})
    assert _relerr(y, ref) <= TOL


def test_contraction_variant_that_does_not_apply_is_refused():
    p = dwm.dwm_plan_create(3, 8, 19, 21, 70, 3, 3, 2, 1)  # reduction padded to 16: no 32- or 64-step chunks
    for v in (11, 12, 13, 14, 15, 16, 18, 19):
        with pytest.raises(dwm.DwmError) as e:
            dwm.dwm_plan_set_variant(p, "contract", v)
        assert e.value.status == dwm.DWM_ERR_INVALID_ARG
    dwm.dwm_plan_destroy(p)


def test_forward_is_deterministic_and_plan_reusable():
    shape = (2, 24, 14, 14, 40, 7, 7, 1, 3)
    x, w = _rand(*shape[:7], seed=9)
    r = Runner(*shape)
    r.set_filter(w)
    y1 = r.forward(x).copy()
    r.y.fill_(float("nan"))
    y2 = r.forward(x).copy()
    x2 = (x * 0.5).astype(np.float32)
    y3 = r.forward(x2)
    assert np.array_equal(y1, y2)
    assert _relerr(y3, oracle.direct_f64(x2, w, 1, 3)) <= TOL
    r.close()


def test_staged_calls_equal_the_fused_entry_point():
    shape = (2, 5, 21, 20, 9, 5, 5, 2, 2)
    x, w = _rand(*shape[:7], seed=10)
    r = Runner(*shape, variants={"forward": 0})
    r.set_filter(w)
    y1 = r.forward(x).copy()
    r.y.fill_(float("nan"))
    dwm.dwm_input_transform(r.plan, r.x.data_ptr(), r.stream())
    dwm.dwm_contract_output(r.plan, r.Ugw.data_ptr(), r.y.data_ptr(), r.stream())
    torch.cuda.synchronize()
    assert np.array_equal(y1, r.y.cpu().numpy())
    r.close()


def test_runs_on_a_side_stream():
    shape = (1, 16, 32, 32, 16, 5, 5, 1, 2)
    x, w = _rand(*shape[:7], seed=13)
    ref = oracle.direct_f64(x, w, 1, 2)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        y = conv(x, w, 1, 2)
    assert _relerr(y, ref) <= TOL


# ---- the five benchmark layers at full size, in the launch configuration bench.py times ----

def test_single_kernel_path_is_chosen_only_where_it_applies():
    few = dwm.dwm_plan_create(2, 3, 40, 40, 8, 7, 7, 2, 3)
    many = dwm.dwm_plan_create(2, 64, 40, 40, 8, 7, 7, 2, 3)
    dwm.dwm_plan_set_variant(few, "forward", 1)
    with pytest.raises(dwm.DwmError):
        dwm.dwm_plan_set_variant(many, "forward", 1)
    dwm.dwm_plan_destroy(few)
    dwm.dwm_plan_destroy(many)


@pytest.mark.parametrize("shape", [(2, 3, 37, 35, 33, 7, 7, 2, 3), (3, 3, 50, 61, 100, 11, 11, 4, 0),
                                   (2, 16, 33, 31, 130, 5, 5, 1, 2), (1, 1, 20, 20, 1, 3, 3, 1, 1),
                                   (2, 5, 150, 140, 70, 3, 3, 2, 1), (1, 8, 20, 24, 40, 7, 1, 1, 3)])
def test_single_kernel_path_matches_fp64_direct(shape):
    """Shapes on which the single-kernel path applies, forced on: K from 1 to beyond one
    workgroup's 128 filters, odd sizes, blocks of tiles that overhang the image."""
    N, C, H, W, K, R, S, s, P = shape
    x, w = _rand(*shape[:7], seed=31)
    ref = oracle.direct_f64(x, w, s, P)
    y = conv(x, w, s, P, variants={"forward": 1})
    assert np.all(np.isfinite(y))
    assert _relerr(y, ref) <= TOL, shape


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_benchmark_layers_full_size(index):
    """Whole layer on the GPU in the launch configuration bench.py times, EVERY output compared with the
    FP64 direct convolution (the oracle takes 1-10 s per layer on the machine's cores)."""
    L = wl.CONFIGS[index]
    x, w = wl.make_layer_tensors(L, index)
    print("forward, whole output:", L.name, flush=True)
    y = conv(x, w, L.stride, L.pad)
    OH, OW = wl.out_hw(L)
    assert y.shape == (L.N, L.K, OH, OW) and np.all(np.isfinite(y))
    ref = oracle.direct_f64(x, w, L.stride, L.pad)
    scale = np.max(np.abs(ref))
    err = np.abs(y - ref)
    worst = np.unravel_index(np.argmax(err), err.shape)
    assert err[worst] / scale <= TOL, (L.name, worst)
    mse = float(np.mean(err ** 2))
    print("%s: max rel err %.3e, MSE %.3e, log10(MSE)+10 = %.2f" % (L.name, err[worst] / scale, mse, np.log10(mse) + 10))


@pytest.mark.parametrize("index", [1, 2])
def test_split_tile_summing_repeats_bit_for_bit(index):
    """The two layers whose contraction cuts tiles into ranges summed across workgroups (and XCDs):
    200 launches on the same input, every y compared on the device with the first, stopping at the
    first mismatch; the first is checked against the oracle by the test above."""
    L = wl.CONFIGS[index]
    x, w = wl.make_layer_tensors(L, index)
    r = Runner(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad)
    try:
        r.set_filter(w)
        r.x = torch.from_numpy(x).cuda()
        args = (r.plan, r.x.data_ptr(), r.Ugw.data_ptr(), r.y.data_ptr(), r.stream())
        dwm.dwm_conv_forward(*args)
        first = r.y.clone()
        assert bool(torch.isfinite(first).all())
        for i in range(200):
            r.y.fill_(float("nan"))
            dwm.dwm_conv_forward(*args)
            assert torch.equal(r.y, first), "launch %d of %s differs from the first" % (i + 1, L.name)
    finally:
        r.close()


@pytest.mark.parametrize("kernel,hw,stride", [(7, 14, 2),    # 256 tiles: every tile cut into two ranges of its own
                                              (3, 28, 1),    # 1568 tiles: three workgroups per CU
                                              (5, 14, 1)])   # 784 tiles, four classes
def test_paper_layers_full_size(kernel, hw, stride):
    """The paper's own single-layer shapes (Sec. 5.1: batch 256, same padding, standard-normal
    inputs and weights) at full size, in the launch configuration the planner picks; the oracle
    computes 20 000 sampled outputs one by one."""
    L = wl.paper_layer(kernel, hw, stride)
    x, w = wl.make_layer_tensors(L, 10 * kernel + stride)
    y = conv(x, w, L.stride, L.pad)
    OH, OW = wl.out_hw(L)
    assert y.shape == (L.N, L.K, OH, OW) and np.all(np.isfinite(y))
    rng = np.random.default_rng(777 + kernel)
    idx = rng.choice(y.size, 20000, replace=False)
    n, k = L.N - 1, L.K - 1
    edge = [((n * L.K + k) * OH + OH - 1) * OW + j for j in range(OW)] + [j for j in range(OW)]
    idx = np.unique(np.concatenate([idx, np.array(edge)]))
    ref = oracle.direct_f64_at(x, w, L.stride, L.pad, idx)
    got = y.ravel()[idx].astype(np.float64)
    assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) <= TOL, L.name
