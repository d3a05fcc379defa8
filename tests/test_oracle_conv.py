"""Pins for the oracle's two convolutions.

O1 (direct FP64) is pinned by closed forms, a pure-Python brute force and the float64
CPU convolution of PyTorch (a library routine, used only here).  O2 (the paper's five
steps in FP64) is pinned by O1: the paper states the aggregated result equals the
regular convolution (Sec. 4.1 "Aggregation"), so the two must agree to rounding.
"""
import numpy as np
import pytest
import torch

import dwm_workloads as wl
import oracle


def _rand(N, C, H, W, K, R, S, seed):
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    return x, w


def _brute(x, w, s, P):
    """Seven nested Python loops over a zero-padded copy (tiny shapes only)."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    xp = np.zeros((N, C, H + 2 * P, W + 2 * P))
    xp[:, :, P:P + H, P:P + W] = x
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    y = np.zeros((N, K, OH, OW))
    for n in range(N):
        for k in range(K):
            for oh in range(OH):
                for ow in range(OW):
                    acc = 0.0
                    for c in range(C):
                        for r in range(R):
                            for q in range(S):
                                acc += xp[n, c, oh * s + r, ow * s + q] * float(w[k, c, r, q])
                    y[n, k, oh, ow] = acc
    return y


def _relerr(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


@pytest.mark.parametrize("R,S,s,P,H,W", [(3, 3, 1, 1, 5, 6), (5, 3, 2, 2, 7, 9), (4, 7, 3, 0, 11, 10),
                                         (1, 1, 2, 0, 5, 5), (2, 2, 1, 1, 3, 4), (11, 11, 4, 0, 19, 23)])
def test_direct_vs_python_brute_force(R, S, s, P, H, W):
    x, w = _rand(2, 3, H, W, 2, R, S, seed=R * 100 + S * 10 + s)
    assert _relerr(oracle.direct_f64(x, w, s, P), _brute(x, w, s, P)) < 1e-14


@pytest.mark.parametrize("R,S,s,P", [(3, 3, 1, 1), (5, 5, 1, 2), (7, 7, 2, 3), (11, 11, 4, 0), (3, 3, 2, 1),
                                     (1, 7, 1, 3), (5, 3, 3, 2), (9, 9, 2, 4), (1, 1, 1, 0), (2, 4, 2, 5)])
def test_direct_vs_library_float64_conv(R, S, s, P):
    x, w = _rand(3, 5, 17, 14, 4, R, S, seed=R + 31 * S + 7 * s)
    want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                      stride=s, padding=P).numpy()
    got = oracle.direct_f64(x, w, s, P)
    assert got.shape == want.shape
    assert _relerr(got, want) < 1e-13


def test_direct_delta_kernel_is_a_strided_shifted_crop():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 1, 12, 13)).astype(np.float32)
    R, S, s, P, r0, q0 = 5, 4, 2, 2, 3, 1
    w = np.zeros((1, 1, R, S), np.float32)
    w[0, 0, r0, q0] = 1.0
    y = oracle.direct_f64(x, w, s, P)
    xp = np.zeros((2, 1, 12 + 2 * P, 13 + 2 * P))
    xp[:, :, P:P + 12, P:P + 13] = x
    OH, OW = y.shape[2:]
    want = xp[:, :, r0:r0 + s * OH:s, q0:q0 + s * OW:s]
    assert np.array_equal(y, want)


def test_direct_all_ones_counts_in_bounds_taps():
    x = np.ones((1, 2, 6, 6), np.float32)
    w = np.ones((1, 2, 3, 3), np.float32)
    y = oracle.direct_f64(x, w, 1, 1)
    assert y[0, 0, 0, 0] == 2 * 4 and y[0, 0, 0, 3] == 2 * 6 and y[0, 0, 2, 2] == 2 * 9
    assert y.sum() == 2 * (16 * 9 + 16 * 6 + 4 * 4)


def test_direct_1x1_is_a_per_pixel_matrix_product():
    x, w = _rand(2, 6, 5, 4, 3, 1, 1, seed=3)
    y = oracle.direct_f64(x, w, 1, 0)
    want = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    assert _relerr(y, want) < 1e-15


def test_direct_at_matches_full():
    x, w = _rand(2, 3, 9, 8, 4, 3, 3, seed=9)
    y = oracle.direct_f64(x, w, 2, 1)
    idx = np.array([0, 5, y.size - 1, 17, 33])
    assert np.array_equal(oracle.direct_f64_at(x, w, 2, 1, idx), y.ravel()[idx])
    with pytest.raises(ValueError):
        oracle.direct_f64_at(x, w, 2, 1, np.array([y.size]))


def test_direct_rejects_bad_shapes():
    x, w = _rand(1, 1, 3, 3, 1, 5, 5, seed=1)
    with pytest.raises(ValueError):
        oracle.direct_f64(x, w, 1, 0)  # kernel larger than the padded input


_SWEEP = [(R, S, s, P) for R in (1, 2, 3, 4, 5, 6, 7, 9, 11) for S in (1, 3, 5, 7, 10)
          for s in (1, 2, 3, 4) for P in (0, 1, 3, 5)]


@pytest.fixture
def f22_form(request):
    oracle.set_f22_form(request.param)
    yield request.param
    oracle.set_f22_form(0)


@pytest.mark.parametrize("f22_form", [0, 1], indirect=True)
def test_dwm_equals_direct_sweep(f22_form):
    """FP64 DWM == direct conv to 1e-12 relative over kernel sizes 1..11 (R != S too),
    strides 1..4, paddings 0..5 (also not multiples of the stride), odd H/W, odd OH/OW;
    with either of the two F(2,2) forms on the 2-tap pieces."""
    worst = 0.0
    for i, (R, S, s, P) in enumerate(_SWEEP):
        H, W = 9 + (i % 5), 8 + (i % 7)
        if H + 2 * P < R or W + 2 * P < S:
            continue
        x, w = _rand(1 + i % 2, 2 + i % 3, H, W, 1 + i % 4, R, S, seed=1000 + i)
        e = _relerr(oracle.dwm_f64(x, w, s, P), oracle.direct_f64(x, w, s, P))
        worst = max(worst, e)
        assert e < 1e-12, (R, S, s, P, H, W, e)
    assert worst > 0.0  # the two paths really are different computations


def test_dwm_equals_direct_on_benchmark_config_1():
    L = wl.CONFIGS[0]
    x, w = wl.make_layer_tensors(L, 0)
    assert _relerr(oracle.dwm_f64(x, w, L.stride, L.pad), oracle.direct_f64(x, w, L.stride, L.pad)) < 1e-12


@pytest.mark.parametrize("R,s,P,H", [(7, 2, 3, 20), (11, 4, 0, 31), (3, 2, 1, 12)])
def test_dwm_equals_direct_on_scaled_down_stem_shapes(R, s, P, H):
    x, w = _rand(2, 3, H, H + 1, 5, R, R, seed=R)
    assert _relerr(oracle.dwm_f64(x, w, s, P), oracle.direct_f64(x, w, s, P)) < 1e-12


@pytest.mark.parametrize("f22_form", [0, 1], indirect=True)
def test_part_stage_functions_compose_to_the_full_result(f22_form):
    """Sum over parts of A^T[(U .* V summed over c)]A, assembled here from the staged
    U and V the oracle exposes, equals O1: pins the stage outputs that the GPU's
    filter- and input-transform kernels are compared against."""
    R = S = 5
    s, P = 2, 2
    x, w = _rand(1, 3, 11, 12, 2, R, S, seed=77)
    y = oracle.direct_f64(x, w, s, P)
    OH, OW = y.shape[2:]
    acc = np.zeros((2, 2 * ((OH + 1) // 2), 2 * ((OW + 1) // 2)))
    for part in oracle.split_2d(R, S, s):
        _, _, AT_h = oracle.winograd_matrices(part[2])
        _, _, AT_w = oracle.winograd_matrices(part[5])
        U = oracle.part_filter_transform(w, s, part)              # [K][C][th][tw]
        V = oracle.part_input_transform(x, R, S, s, P, part, 0)   # [C][TH][TW][th][tw]
        M = np.einsum("kcij,cyxij->kyxij", U, V)
        Y = np.einsum("ai,kyxij,bj->kyaxb", AT_h, M, AT_w)
        acc += Y.reshape(2, acc.shape[1], acc.shape[2])
    assert _relerr(acc[:, :OH, :OW], y[0]) < 1e-13


def test_mse_report_form():
    """log10(MSE)+10 (Fig. 1b caption): an MSE of 1e-10 reports as 0."""
    ref = np.zeros(4)
    ref[0] = 2.0
    mse, rep, rel = oracle.mse_report(ref + 1e-5, ref)
    assert abs(mse - 1e-10) < 1e-16 and abs(rep - 0.0) < 1e-6 and abs(rel - 0.5e-5) < 1e-12
