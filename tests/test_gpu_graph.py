"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation,
no memset): a forward call (single or half precision), and either gradient, can therefore be captured into a HIP graph and replayed.  Every replay
is checked against the eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

import paper_2002_00552_amd as dwm

pytestmark = pytest.mark.gpu


def _setup(shape, forward_variant):
    N, C, H, W, K, R, S, s, P = shape
    rng = np.random.default_rng(5)
    x = torch.from_numpy(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)).cuda()
    w = torch.from_numpy((rng.standard_normal((K, C, R, S)) * np.sqrt(2.0 / (C * R * S))).astype(np.float32)).cuda()
    plan = dwm.dwm_plan_create(N, C, H, W, K, R, S, s, P)
    if forward_variant is not None:
        dwm.dwm_plan_set_variant(plan, "forward", forward_variant)
    info = dwm.dwm_plan_info(plan)
    U = torch.empty(dwm.dwm_plan_filter_bytes(plan) // 4, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(dwm.dwm_plan_workspace_bytes(plan) // 4, 64), dtype=torch.float32, device="cuda")
    dwm.dwm_plan_set_workspace(plan, ws.data_ptr(), ws.numel() * 4)
    y = torch.zeros((N, K, info.OH, info.OW), dtype=torch.float32, device="cuda")
    return plan, x, w, U, ws, y


@pytest.mark.parametrize("shape,forward_variant", [
    ((1, 16, 32, 32, 16, 5, 5, 1, 2), None),   # single-kernel path
    ((1, 16, 32, 32, 16, 5, 5, 1, 2), 0),      # staged path with split tiles (arrival counters)
    ((2, 64, 30, 30, 64, 3, 3, 1, 1), 0),      # staged path, whole and split tiles
])
def test_forward_replays_from_a_graph(shape, forward_variant):
    plan, x, w, U, ws, y = _setup(shape, forward_variant)
    try:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            st = side.cuda_stream
            dwm.dwm_filter_transform(plan, w.data_ptr(), U.data_ptr(), st)
            dwm.dwm_conv_forward(plan, x.data_ptr(), U.data_ptr(), y.data_ptr(), st)  # eager, also warms up
            side.synchronize()
            eager = y.clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                dwm.dwm_conv_forward(plan, x.data_ptr(), U.data_ptr(), y.data_ptr(), torch.cuda.current_stream().cuda_stream)
        for rep in range(4):
            y.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, eager), "replay %d" % rep
            # eager work between replays, on another input, through the same plan and workspace
            x2 = x * 0.5
            dwm.dwm_conv_forward(plan, x2.data_ptr(), U.data_ptr(), y.data_ptr(), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert not torch.equal(y, eager)
    finally:
        torch.cuda.synchronize()
        dwm.dwm_plan_destroy(plan)


def _replay_and_compare(g, out, eager, eager_again):
    """Four replays, each checked against the eager result, with eager work on other data and
    synchronisations in between."""
    for rep in range(4):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d" % rep
        eager_again()
        torch.cuda.synchronize()
        assert not torch.equal(out, eager)


@pytest.mark.parametrize("shape", [
    (2, 10, 20, 24, 150, 3, 3, 2, 1),    # four sub-convolutions, one merged input transform, one batched contraction
    (2, 24, 14, 14, 40, 7, 7, 1, 3),     # one sub-convolution on the forward kernels (tiles cut into ranges)
    (2, 3, 37, 35, 33, 7, 7, 2, 3),      # three channels: the whole gradient in one kernel
])
def test_backward_data_replays_from_a_graph(shape):
    N, C, H, W, K, R, S, s, P = shape
    rng = np.random.default_rng(6)
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    w = torch.from_numpy((rng.standard_normal((K, C, R, S)) * 0.1).astype(np.float32)).cuda()
    dy = torch.from_numpy(rng.uniform(-1, 1, (N, K, OH, OW)).astype(np.float32)).cuda()
    plan = dwm.dwm_bwd_data_plan_create(N, C, H, W, K, R, S, s, P)
    try:
        U = torch.empty(dwm.dwm_bwd_data_filter_bytes(plan) // 4, dtype=torch.float32, device="cuda")
        ws = torch.empty(max(dwm.dwm_bwd_data_workspace_bytes(plan) // 4, 64), dtype=torch.float32, device="cuda")
        dwm.dwm_bwd_data_set_workspace(plan, ws.data_ptr(), ws.numel() * 4)
        dx = torch.zeros((N, C, H, W), dtype=torch.float32, device="cuda")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            st = side.cuda_stream
            dwm.dwm_bwd_data_filter_transform(plan, w.data_ptr(), U.data_ptr(), st)
            dwm.dwm_conv_backward_data(plan, dy.data_ptr(), U.data_ptr(), dx.data_ptr(), st)
            side.synchronize()
            eager = dx.clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                dwm.dwm_conv_backward_data(plan, dy.data_ptr(), U.data_ptr(), dx.data_ptr(),
                                           torch.cuda.current_stream().cuda_stream)
        dy2 = dy * 0.5
        _replay_and_compare(g, dx, eager, lambda: dwm.dwm_conv_backward_data(
            plan, dy2.data_ptr(), U.data_ptr(), dx.data_ptr(), torch.cuda.current_stream().cuda_stream))
    finally:
        torch.cuda.synchronize()
        dwm.dwm_bwd_data_plan_destroy(plan)


@pytest.mark.parametrize("shape", [
    (2, 66, 12, 12, 67, 3, 3, 1, 1),     # GEMM form: input transform, dy transform, GEMM over ranges, final
    (16, 6, 130, 127, 16, 3, 3, 2, 1),   # short-reduction form: class kernels in one launch, reduce, final
])
def test_backward_filter_replays_from_a_graph(shape):
    N, C, H, W, K, R, S, s, P = shape
    rng = np.random.default_rng(7)
    OH, OW = (H + 2 * P - R) // s + 1, (W + 2 * P - S) // s + 1
    x = torch.from_numpy(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)).cuda()
    dy = torch.from_numpy(rng.uniform(-1, 1, (N, K, OH, OW)).astype(np.float32)).cuda()
    plan = dwm.dwm_bwd_filter_plan_create(N, C, H, W, K, R, S, s, P)
    try:
        ws = torch.empty(dwm.dwm_bwd_filter_workspace_bytes(plan) // 4, dtype=torch.float32, device="cuda")
        dwm.dwm_bwd_filter_set_workspace(plan, ws.data_ptr(), ws.numel() * 4)
        dw = torch.zeros((K, C, R, S), dtype=torch.float32, device="cuda")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            st = side.cuda_stream
            dwm.dwm_conv_backward_filter(plan, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), st)
            side.synchronize()
            eager = dw.clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                dwm.dwm_conv_backward_filter(plan, x.data_ptr(), dy.data_ptr(), dw.data_ptr(),
                                             torch.cuda.current_stream().cuda_stream)
        dy2 = dy * 0.5
        _replay_and_compare(g, dw, eager, lambda: dwm.dwm_conv_backward_filter(
            plan, x.data_ptr(), dy2.data_ptr(), dw.data_ptr(), torch.cuda.current_stream().cuda_stream))
    finally:
        torch.cuda.synchronize()
        dwm.dwm_bwd_filter_plan_destroy(plan)


@pytest.mark.parametrize("shape", [
    (2, 64, 30, 30, 64, 3, 3, 1, 1),     # LDS-staged input transform, whole and split tiles
    (2, 3, 37, 35, 33, 7, 7, 2, 3),      # three channels: the 16-bit single kernel
    (2, 24, 14, 14, 40, 7, 7, 1, 3),     # 24 channels: eight-row items of the LDS-staged input transform
])
def test_half_precision_forward_replays_from_a_graph(shape):
    N, C, H, W, K, R, S, s, P = shape
    rng = np.random.default_rng(8)
    x = torch.from_numpy(rng.uniform(-1, 1, (N, C, H, W)).astype(np.float16)).cuda()
    w = torch.from_numpy((rng.standard_normal((K, C, R, S)) * 0.1).astype(np.float16)).cuda()
    plan = dwm.dwm_f16_plan_create(N, C, H, W, K, R, S, s, P)
    try:
        info = dwm.dwm_f16_plan_info(plan)
        U = torch.empty(dwm.dwm_f16_filter_bytes(plan) // 2, dtype=torch.float16, device="cuda")
        ws = torch.empty(max(dwm.dwm_f16_workspace_bytes(plan), 256), dtype=torch.uint8, device="cuda")
        dwm.dwm_f16_set_workspace(plan, ws.data_ptr(), ws.numel())
        y = torch.zeros((N, K, info.OH, info.OW), dtype=torch.float16, device="cuda")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            st = side.cuda_stream
            dwm.dwm_f16_filter_transform(plan, w.data_ptr(), U.data_ptr(), st)
            dwm.dwm_f16_conv_forward(plan, x.data_ptr(), U.data_ptr(), y.data_ptr(), st)
            side.synchronize()
            eager = y.clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                dwm.dwm_f16_conv_forward(plan, x.data_ptr(), U.data_ptr(), y.data_ptr(),
                                         torch.cuda.current_stream().cuda_stream)
        x2 = x * 0.5
        _replay_and_compare(g, y, eager, lambda: dwm.dwm_f16_conv_forward(
            plan, x2.data_ptr(), U.data_ptr(), y.data_ptr(), torch.cuda.current_stream().cuda_stream))
    finally:
        torch.cuda.synchronize()
        dwm.dwm_f16_plan_destroy(plan)
