"""Pins for the oracle's gradients with respect to the input and to the filter.

O1' (the definition of dL/dx) is pinned by the adjoint identity against the pinned forward
oracle O1, by PyTorch's float64 autograd on CPU (a library routine, used only here), by a
pure-Python scatter brute force and by a closed form.  O2' (the paper's backward formulas,
Sec. 3.1 eq. 5 and Sec. 4.2 eq. 16-17) is pinned by O1'.
"""
import numpy as np
import pytest
import torch

import oracle


def _rand(N, C, H, W, K, R, S, s, P, seed):
    rng = np.random.default_rng(seed)
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    dy = rng.standard_normal((N, K, OH, OW)).astype(np.float32)
    return x, w, dy


def _relerr(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


SHAPES = [(3, 3, 1, 1, 6, 7), (5, 3, 2, 2, 9, 8), (7, 7, 2, 3, 13, 12), (11, 11, 4, 0, 23, 25), (1, 1, 2, 0, 5, 6),
          (4, 6, 3, 2, 11, 13), (2, 2, 2, 0, 8, 8), (3, 3, 2, 1, 8, 9), (1, 7, 1, 3, 5, 9), (5, 5, 1, 0, 9, 9),
          (3, 3, 4, 1, 10, 11), (2, 3, 3, 5, 7, 6)]


@pytest.mark.parametrize("R,S,s,P,H,W", SHAPES)
def test_backward_data_is_the_adjoint_of_the_forward_oracle(R, S, s, P, H, W):
    """<dy, conv(x, w)> == <dL/dx, x> for arbitrary x and dy: the defining property."""
    x, w, dy = _rand(2, 3, H, W, 4, R, S, s, P, seed=R * 100 + S * 10 + s)
    y = oracle.direct_f64(x, w, s, P)
    dx = oracle.backward_data_f64(dy, w, x.shape, s, P)
    lhs, rhs = float(np.sum(dy.astype(np.float64) * y)), float(np.sum(dx * x.astype(np.float64)))
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), np.sum(np.abs(dx * x)))
    # and pixel by pixel: the gradient is the response to a one-hot x
    rng = np.random.default_rng(1)
    for _ in range(5):
        n, c, ih, iw = rng.integers(2), rng.integers(3), rng.integers(H), rng.integers(W)
        e = np.zeros_like(x)
        e[n, c, ih, iw] = 1.0
        want = float(np.sum(dy.astype(np.float64) * oracle.direct_f64(e, w, s, P)))
        assert abs(dx[n, c, ih, iw] - want) <= 1e-12 * max(1.0, abs(want))


@pytest.mark.parametrize("R,S,s,P,H,W", SHAPES)
def test_backward_data_vs_library_autograd(R, S, s, P, H, W):
    x, w, dy = _rand(2, 3, H, W, 4, R, S, s, P, seed=7 + R + S + s)
    xt = torch.from_numpy(x).double().requires_grad_(True)
    yt = torch.nn.functional.conv2d(xt, torch.from_numpy(w).double(), stride=s, padding=P)
    yt.backward(torch.from_numpy(dy).double())
    got = oracle.backward_data_f64(dy, w, x.shape, s, P)
    assert _relerr(got, xt.grad.numpy()) < 1e-13


@pytest.mark.parametrize("R,S,s,P,H,W", [(3, 3, 1, 1, 5, 6), (5, 3, 2, 2, 7, 9), (4, 4, 3, 0, 10, 11)])
def test_backward_data_vs_python_scatter(R, S, s, P, H, W):
    """Every output pixel pushes dy * w back onto the window it was computed from."""
    x, w, dy = _rand(1, 2, H, W, 2, R, S, s, P, seed=3)
    N, K, OH, OW = dy.shape
    C = w.shape[1]
    gp = np.zeros((N, C, H + 2 * P, W + 2 * P))
    for n in range(N):
        for k in range(K):
            for oh in range(OH):
                for ow in range(OW):
                    for c in range(C):
                        for r in range(R):
                            for q in range(S):
                                gp[n, c, oh * s + r, ow * s + q] += float(dy[n, k, oh, ow]) * float(w[k, c, r, q])
    want = gp[:, :, P:P + H, P:P + W]
    assert _relerr(oracle.backward_data_f64(dy, w, x.shape, s, P), want) < 1e-14


def test_backward_data_of_a_delta_kernel_is_a_strided_placement():
    """One tap at (r0, q0): dx[ih, iw] = dy[(ih+P-r0)/s, (iw+P-q0)/s] where that is an integer
    output position, zero elsewhere (also: pixels no window touches get a zero gradient)."""
    rng = np.random.default_rng(9)
    H, W, R, S, s, P, r0, q0 = 12, 13, 4, 3, 3, 1, 2, 1
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    dy = rng.standard_normal((1, 1, OH, OW)).astype(np.float32)
    w = np.zeros((1, 1, R, S), np.float32)
    w[0, 0, r0, q0] = 1.0
    dx = oracle.backward_data_f64(dy, w, (1, 1, H, W), s, P)
    want = np.zeros((H, W))
    for oh in range(OH):
        for ow in range(OW):
            ih, iw = oh * s + r0 - P, ow * s + q0 - P
            if 0 <= ih < H and 0 <= iw < W:
                want[ih, iw] = dy[0, 0, oh, ow]
    assert np.array_equal(dx[0, 0], want)


def test_backward_data_at_matches_full():
    x, w, dy = _rand(2, 3, 11, 12, 4, 5, 3, 2, 2, seed=21)
    full = oracle.backward_data_f64(dy, w, x.shape, 2, 2)
    idx = np.random.default_rng(0).choice(full.size, 200, replace=False)
    assert np.array_equal(oracle.backward_data_f64_at(dy, w, x.shape, 2, 2, idx), full.ravel()[idx])
    with pytest.raises(ValueError):
        oracle.backward_data_f64_at(dy, w, x.shape, 2, 2, np.array([full.size]))


@pytest.fixture
def f22_form(request):
    oracle.set_f22_form(request.param)
    yield request.param
    oracle.set_f22_form(0)


@pytest.mark.parametrize("f22_form", [0, 1], indirect=True)
def test_paper_backward_formulas_equal_the_definition(f22_form):
    """O2' == O1' to 1e-12 over kernel sizes 1..11, strides 1..4, paddings, odd sizes."""
    worst, i = 0.0, 0
    for R in (1, 2, 3, 5, 7, 11):
        for S in (1, 3, 4, 7):
            for s in (1, 2, 3, 4):
                for P in (0, 1, 3):
                    i += 1
                    H, W = 9 + i % 5, 8 + i % 7
                    if H + 2 * P < R or W + 2 * P < S:
                        continue
                    x, w, dy = _rand(1 + i % 2, 2 + i % 3, H, W, 1 + i % 3, R, S, s, P, seed=500 + i)
                    e = _relerr(oracle.dwm_backward_data_f64(dy, w, x.shape, s, P),
                                oracle.backward_data_f64(dy, w, x.shape, s, P))
                    worst = max(worst, e)
                    assert e < 1e-12, (R, S, s, P, H, W, e)
    assert worst > 0.0


# ---- gradient with respect to the filter ----

@pytest.mark.parametrize("R,S,s,P,H,W", SHAPES)
def test_backward_filter_is_the_adjoint_in_w(R, S, s, P, H, W):
    """conv is linear in w: <dy, conv(x, w)> == <dL/dw, w>, and tap by tap dL/dw is the
    response to a one-hot filter."""
    x, w, dy = _rand(2, 3, H, W, 4, R, S, s, P, seed=40 + R * 100 + S * 10 + s)
    dw = oracle.backward_filter_f64(x, dy, w.shape, s, P)
    lhs = float(np.sum(dy.astype(np.float64) * oracle.direct_f64(x, w, s, P)))
    rhs = float(np.sum(dw * w.astype(np.float64)))
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), np.sum(np.abs(dw * w)))
    rng = np.random.default_rng(2)
    for _ in range(5):
        k, c, r, q = rng.integers(4), rng.integers(3), rng.integers(R), rng.integers(S)
        e = np.zeros_like(w)
        e[k, c, r, q] = 1.0
        want = float(np.sum(dy.astype(np.float64) * oracle.direct_f64(x, e, s, P)))
        assert abs(dw[k, c, r, q] - want) <= 1e-12 * max(1.0, abs(want))


@pytest.mark.parametrize("R,S,s,P,H,W", SHAPES)
def test_backward_filter_vs_library_autograd(R, S, s, P, H, W):
    x, w, dy = _rand(2, 3, H, W, 4, R, S, s, P, seed=77 + R + S + s)
    wt = torch.from_numpy(w).double().requires_grad_(True)
    yt = torch.nn.functional.conv2d(torch.from_numpy(x).double(), wt, stride=s, padding=P)
    yt.backward(torch.from_numpy(dy).double())
    assert _relerr(oracle.backward_filter_f64(x, dy, w.shape, s, P), wt.grad.numpy()) < 1e-13


@pytest.mark.parametrize("f22_form", [0, 1], indirect=True)
def test_paper_filter_gradient_formula_equals_the_definition(f22_form):
    worst, i = 0.0, 0
    for R in (1, 2, 3, 5, 7, 11):
        for S in (1, 3, 4, 7):
            for s in (1, 2, 3, 4):
                for P in (0, 1, 3):
                    i += 1
                    H, W = 9 + i % 5, 8 + i % 7
                    if H + 2 * P < R or W + 2 * P < S:
                        continue
                    x, w, dy = _rand(1 + i % 2, 2 + i % 3, H, W, 1 + i % 3, R, S, s, P, seed=900 + i)
                    e = _relerr(oracle.dwm_backward_filter_f64(x, dy, w.shape, s, P),
                                oracle.backward_filter_f64(x, dy, w.shape, s, P))
                    worst = max(worst, e)
                    assert e < 1e-12, (R, S, s, P, H, W, e)
    assert worst > 0.0
