"""FP64 CPU oracle for the DWM forward convolution -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It never touches the GPU library and shares no code with it.

The arithmetic lives in ``dwm_oracle.c`` (plain C, double precision); this module
compiles it with gcc on first use and exposes thin numpy wrappers:

* ``direct_f64``            O1, the definition of the convolution (ground truth)
* ``direct_f64_at``         O1 at sampled output positions
* ``dwm_f64``               O2, the paper's five steps in FP64
* ``dwm_half_f64``          O2 with binary16 storage of x, w, U and V (Table 1, "DWM FP16")
* ``round_binary16``        nearest binary16 value of each double (ties to even)
* ``backward_data_f64``     O1', the gradient with respect to the input, by definition
* ``dwm_backward_data_f64`` O2', the same by the paper's backward formulas
* ``backward_filter_f64``   O1'', the gradient with respect to the filter, by definition
* ``dwm_backward_filter_f64`` O2'', the same by the paper's formula
* ``split_1d / split_2d``   the paper's kernel splitting (Sec. 4.1, eq. 8 and eq. 12)
* ``mults_per_tile``        the multiplication-count model behind Table 3
* ``winograd_matrices``     B^T, G, A^T of F(2,l), l = 1..3 (Sec. 3.2 for l = 3)
* ``set_f22_form``          which of the two F(2,2) forms the 2-tap pieces use
* ``winograd_1d``           Y = A^T[(G g) .* (B^T d)] (Sec. 3.1)
* ``part_filter_transform`` U = G g G^T of one part
* ``part_input_transform``  V = B^T d B of one part, one image
* ``mse_report``            MSE and the paper's log10(MSE)+10 form (Fig. 1b caption)
"""
import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dwm_oracle.c")
_LIB = os.path.join(_HERE, "libdwm_oracle.so")
_lib = None


def build(force=False):
    """Compile dwm_oracle.c into libdwm_oracle.so with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Part(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("ph", "jh", "lh", "pw", "jw", "lw")]


class _Piece(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("p", "j", "l")]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_mults_per_tile.restype = ctypes.c_longlong
    return _lib


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("oracle inputs are the float32 arrays the GPU sees")
    return a


def out_size(H, R, s, P):
    return (H + 2 * P - R) // s + 1


def num_threads():
    return int(_load().oracle_num_threads())


def direct_f64(x, w, stride, pad):
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    y = np.empty((N, K, out_size(H, R, stride, pad), out_size(W, S, stride, pad)), np.float64)
    rc = _load().oracle_direct_f64(_fp(x), _fp(w), _dp(y), N, C, H, W, K, R, S, stride, pad)
    if rc:
        raise ValueError("oracle_direct_f64: bad shape (rc=%d)" % rc)
    return y


def direct_f64_at(x, w, stride, pad, flat_idx):
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.shape, np.float64)
    rc = _load().oracle_direct_f64_at(
        _fp(x), _fp(w), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_longlong)),
        ctypes.c_longlong(idx.size), _dp(out), N, C, H, W, K, R, S, stride, pad)
    if rc:
        raise ValueError("oracle_direct_f64_at: bad shape or index (rc=%d)" % rc)
    return out


def dwm_f64(x, w, stride, pad):
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    y = np.empty((N, K, out_size(H, R, stride, pad), out_size(W, S, stride, pad)), np.float64)
    rc = _load().oracle_dwm_f64(_fp(x), _fp(w), _dp(y), N, C, H, W, K, R, S, stride, pad)
    if rc:
        raise ValueError("oracle_dwm_f64: bad shape (rc=%d)" % rc)
    return y


def round_binary16(a):
    """Each double rounded to the nearest IEEE binary16 value (ties to even), as float64."""
    a = np.ascontiguousarray(a, np.float64)
    out = np.empty_like(a)
    _load().oracle_round_binary16(_dp(a), _dp(out), ctypes.c_longlong(a.size))
    return out


def dwm_half_f64(x, w, stride, pad):
    """O2 with half-precision storage: x and w hold binary16 values (float16 arrays, or float32
    arrays of such values); U and V are rounded to binary16 before the products; sums in FP64;
    the FP64 result is returned unrounded."""
    x = _f32(np.asarray(x).astype(np.float32))
    w = _f32(np.asarray(w).astype(np.float32))
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    y = np.empty((N, K, out_size(H, R, stride, pad), out_size(W, S, stride, pad)), np.float64)
    rc = _load().oracle_dwm_half_f64(_fp(x), _fp(w), _dp(y), N, C, H, W, K, R, S, stride, pad)
    if rc == 3:
        raise ValueError("oracle_dwm_half_f64: x and w must hold binary16 values")
    if rc:
        raise ValueError("oracle_dwm_half_f64: bad shape (rc=%d)" % rc)
    return y


def round_bfloat16(a):
    """Each double rounded to the nearest bfloat16 value (ties to even), as float64."""
    a = np.ascontiguousarray(a, np.float64)
    out = np.empty_like(a)
    _load().oracle_round_bfloat16(_dp(a), _dp(out), ctypes.c_longlong(a.size))
    return out


def dwm_bf16_f64(x, w, stride, pad):
    """O2 with bfloat16 storage: x and w are float32 arrays holding bfloat16 values; U and V are
    rounded to bfloat16 before the products; sums in FP64; the FP64 result is returned unrounded."""
    x = _f32(np.asarray(x).astype(np.float32))
    w = _f32(np.asarray(w).astype(np.float32))
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    y = np.empty((N, K, out_size(H, R, stride, pad), out_size(W, S, stride, pad)), np.float64)
    rc = _load().oracle_dwm_bf16_f64(_fp(x), _fp(w), _dp(y), N, C, H, W, K, R, S, stride, pad)
    if rc == 3:
        raise ValueError("oracle_dwm_bf16_f64: x and w must hold bfloat16 values")
    if rc:
        raise ValueError("oracle_dwm_bf16_f64: bad shape (rc=%d)" % rc)
    return y


def _bwd(fn, dy, w, x_shape, stride, pad):
    dy, w = _f32(dy), _f32(w)
    N, C, H, W = x_shape
    K, C2, R, S = w.shape
    assert C == C2 and dy.shape == (N, K, out_size(H, R, stride, pad), out_size(W, S, stride, pad))
    dx = np.empty((N, C, H, W), np.float64)
    rc = fn(_fp(dy), _fp(w), _dp(dx), N, C, H, W, K, R, S, stride, pad)
    if rc:
        raise ValueError("backward data: bad shape (rc=%d)" % rc)
    return dx


def backward_data_f64(dy, w, x_shape, stride, pad):
    """O1': dL/dx for L = <dy, conv(x, w)>, by its definition (the paper's backward pass,
    Sec. 3.1 eq. 5 / Sec. 4.2 eq. 16-17, computes this quantity)."""
    return _bwd(_load().oracle_backward_data_f64, dy, w, x_shape, stride, pad)


def backward_data_f64_at(dy, w, x_shape, stride, pad, flat_idx):
    """O1' at sampled positions (flat indices into dx[N][C][H][W])."""
    dy, w = _f32(dy), _f32(w)
    N, C, H, W = x_shape
    K, C2, R, S = w.shape
    assert C == C2 and dy.shape == (N, K, out_size(H, R, stride, pad), out_size(W, S, stride, pad))
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.shape, np.float64)
    rc = _load().oracle_backward_data_f64_at(
        _fp(dy), _fp(w), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_longlong)), ctypes.c_longlong(idx.size),
        _dp(out), N, C, H, W, K, R, S, stride, pad)
    if rc:
        raise ValueError("oracle_backward_data_f64_at: bad shape or index (rc=%d)" % rc)
    return out


def dwm_backward_data_f64(dy, w, x_shape, stride, pad):
    """O2': the same gradient by the paper's formulas, part by part."""
    return _bwd(_load().oracle_dwm_backward_data_f64, dy, w, x_shape, stride, pad)


def _bwd_w(fn, x, dy, w_shape, stride, pad):
    x, dy = _f32(x), _f32(dy)
    N, C, H, W = x.shape
    K, C2, R, S = w_shape
    assert C == C2 and dy.shape == (N, K, out_size(H, R, stride, pad), out_size(W, S, stride, pad))
    dw = np.empty((K, C, R, S), np.float64)
    rc = fn(_fp(x), _fp(dy), _dp(dw), N, C, H, W, K, R, S, stride, pad)
    if rc:
        raise ValueError("backward filter: bad shape (rc=%d)" % rc)
    return dw


def backward_filter_f64(x, dy, w_shape, stride, pad):
    """O1'': dL/dw for L = <dy, conv(x, w)>, by its definition (Sec. 3.1 eq. 5 / Sec. 4.2 eq. 18
    compute this quantity)."""
    return _bwd_w(_load().oracle_backward_filter_f64, x, dy, w_shape, stride, pad)


def dwm_backward_filter_f64(x, dy, w_shape, stride, pad):
    """O2'': the same gradient by the paper's formula, part by part."""
    return _bwd_w(_load().oracle_dwm_backward_filter_f64, x, dy, w_shape, stride, pad)


def split_1d(r, s):
    """[(phase, offset, length)] of a length-r 1-D kernel at stride s."""
    buf = (_Piece * 64)()
    n = _load().oracle_split_1d(r, s, buf, 64)
    if n < 0:
        raise ValueError("too many pieces")
    return [(buf[i].p, buf[i].j, buf[i].l) for i in range(n)]


def split_2d(R, S, s):
    """[(ph, jh, lh, pw, jw, lw)] of an R x S kernel at stride s."""
    buf = (_Part * 4096)()
    n = _load().oracle_split_2d(R, S, s, buf, 4096)
    if n < 0:
        raise ValueError("too many parts")
    return [(b.ph, b.jh, b.lh, b.pw, b.jw, b.lw) for b in buf[:n]]


def mults_per_tile(R, S, s):
    return int(_load().oracle_mults_per_tile(R, S, s))


def set_f22_form(form):
    """Which three-multiplication F(2,2) every function below uses for 2-tap pieces:
    0 = the form with entries 0/+-1 (default), 1 = the printed F(2,3) without its point at
    infinity (points 0, 1, -1).  The paper prints neither; both are exact."""
    if _load().oracle_set_f22_form(int(form)):
        raise ValueError("form must be 0 or 1")


def winograd_matrices(l):
    t = l + 1
    BT, G, AT = np.zeros((t, t)), np.zeros((t, l)), np.zeros((2, t))
    if _load().oracle_winograd_matrices(l, _dp(BT), _dp(G), _dp(AT)):
        raise ValueError("l must be 1, 2 or 3")
    return BT, G, AT


def winograd_1d(g, d):
    g = np.ascontiguousarray(g, np.float64)
    d = np.ascontiguousarray(d, np.float64)
    l = g.size
    assert d.size == l + 1
    y = np.zeros(2)
    if _load().oracle_winograd_1d(l, _dp(g), _dp(d), _dp(y)):
        raise ValueError("l must be 1, 2 or 3")
    return y


def part_filter_transform(w, stride, part):
    """U[K][C][lh+1][lw+1] of one part (ph, jh, lh, pw, jw, lw)."""
    w = _f32(w)
    K, C, R, S = w.shape
    pt = _Part(*part)
    U = np.empty((K, C, pt.lh + 1, pt.lw + 1), np.float64)
    if _load().oracle_part_filter_transform(_fp(w), K, C, R, S, stride, ctypes.byref(pt), _dp(U)):
        raise ValueError("part reaches outside the kernel")
    return U


def part_input_transform(x, R, S, stride, pad, part, n):
    """V[C][TH][TW][lh+1][lw+1] of one part for image n."""
    x = _f32(x)
    N, C, H, W = x.shape
    OH, OW = out_size(H, R, stride, pad), out_size(W, S, stride, pad)
    TH, TW = (OH + 1) // 2, (OW + 1) // 2
    pt = _Part(*part)
    V = np.empty((C, TH, TW, pt.lh + 1, pt.lw + 1), np.float64)
    _load().oracle_part_input_transform(_fp(x), C, H, W, stride, pad, TH, TW, n, ctypes.byref(pt), _dp(V))
    return V


def mse_report(y_test, y_ref64):
    """(mse, log10(mse)+10, max|diff|/max|y_ref|): the paper reports accuracy as the
    MSE against the FP64 convolution, plotted as log10(MSE)+10 (Fig. 1b caption)."""
    d = np.asarray(y_test, np.float64) - y_ref64
    mse = float(np.mean(d * d))
    rep = math.log10(mse) + 10.0 if mse > 0 else float("-inf")
    scale = float(np.max(np.abs(y_ref64)))
    rel = float(np.max(np.abs(d))) / scale if scale > 0 else float(np.max(np.abs(d)))
    return mse, rep, rel
