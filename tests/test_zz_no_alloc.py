"""dwm_conv_forward_static (the entry point that allocates nothing) against dwm_conv_forward.

Two calls in a row on the library's own scratch array, the second on a smaller layer: the second
must not see anything the first left behind.  Both are compared bit for bit with the existing
entry point (same kernels, same launch shapes) and, to the parity bar, with the FP64 definition.
"""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2002_00552_amd as dwm

pytestmark = pytest.mark.gpu

# (N, C, H, W, K, R, S, stride, pad): many channels, so the staged path (V in the scratch array) runs;
# the first has split tiles (partial outputs and arrival counters in the scratch array as well)
LAYERS = [(3, 96, 30, 30, 80, 5, 5, 1, 2), (1, 72, 13, 17, 40, 3, 3, 2, 1)]


def _run(shape, seed, static):
    import torch
    N, C, H, W, K, R, S, s, P = shape
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)
    plan = dwm.dwm_plan_create(*shape)
    try:
        dwm.dwm_plan_set_variant(plan, "forward", 0)
        info = dwm.dwm_plan_info(plan)
        assert info.forward_path == 0
        need = dwm.dwm_plan_workspace_bytes(plan)
        assert need <= dwm.dwm_static_scratch_bytes()
        xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        U = torch.empty(dwm.dwm_plan_filter_bytes(plan) // 4, dtype=torch.float32, device="cuda")
        y = torch.full((N, K, info.OH, info.OW), float("nan"), dtype=torch.float32, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        dwm.dwm_filter_transform(plan, wd.data_ptr(), U.data_ptr(), st)
        if static:
            dwm.dwm_conv_forward_static(plan, xd.data_ptr(), U.data_ptr(), y.data_ptr(), st)
        else:
            ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")
            dwm.dwm_plan_set_workspace(plan, ws.data_ptr(), need)
            dwm.dwm_conv_forward(plan, xd.data_ptr(), U.data_ptr(), y.data_ptr(), st)
        torch.cuda.synchronize()
        return x, w, y.cpu().numpy()
    finally:
        dwm.dwm_plan_destroy(plan)


def test_static_scratch_forward_two_calls():
    outs = []
    for i, shape in enumerate(LAYERS):  # the larger layer first, then the smaller one on the same array
        print("static forward", shape, flush=True)
        outs.append(_run(shape, 50 + i, static=True))
    for i, shape in enumerate(LAYERS):
        x, w, got = outs[i]
        _, _, want = _run(shape, 50 + i, static=False)
        assert np.array_equal(got, want), shape
        ref = oracle.direct_f64(x, w, shape[7], shape[8])
        assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) <= 1e-4, shape


def test_static_scratch_limit_and_arguments():
    L = dwm.lib()
    assert dwm.dwm_static_scratch_bytes() == 32 << 20
    # a layer whose transformed input alone outgrows the array is refused, nothing is launched
    plan = dwm.dwm_plan_create(32, 128, 56, 56, 256, 3, 3, 2, 1)
    try:
        assert dwm.dwm_plan_workspace_bytes(plan) > dwm.dwm_static_scratch_bytes()
        one = ctypes.c_void_p(256)
        assert L.dwm_conv_forward_static(plan, one, one, one, None) == dwm.DWM_ERR_WORKSPACE
        assert L.dwm_conv_forward_static(plan, None, one, one, None) == dwm.DWM_ERR_INVALID_ARG
        assert L.dwm_conv_forward_static(None, one, one, one, None) == dwm.DWM_ERR_INVALID_ARG
    finally:
        dwm.dwm_plan_destroy(plan)
