"""Helpers for the GPU tests: run the library through its C ABI on torch device buffers."""
import numpy as np
import torch

import paper_2002_00552_amd as dwm


class Runner:
    """One plan with its device buffers; PyTorch supplies memory and the stream only."""

    def __init__(self, N, C, H, W, K, R, S, stride, pad, variants=None):
        self.plan = dwm.dwm_plan_create(N, C, H, W, K, R, S, stride, pad)
        self.info = dwm.dwm_plan_info(self.plan)
        dev = torch.device("cuda:0")
        for stage, v in (variants or {}).items():  # before sizing: the workspace depends on the variant
            dwm.dwm_plan_set_variant(self.plan, stage, v)
        self.Ugw = torch.empty(dwm.dwm_plan_filter_bytes(self.plan) // 4, dtype=torch.float32, device=dev)
        # poison the workspace so that anything the input transform fails to write shows up
        self.ws = torch.full((max(dwm.dwm_plan_workspace_bytes(self.plan) // 4, 1),), float("nan"),
                             dtype=torch.float32, device=dev)
        dwm.dwm_plan_set_workspace(self.plan, self.ws.data_ptr(), self.ws.numel() * 4)
        self.y = torch.full((N, K, self.info.OH, self.info.OW), float("nan"), dtype=torch.float32, device=dev)

    def stream(self):
        return torch.cuda.current_stream().cuda_stream

    def set_filter(self, w):
        self.w = torch.from_numpy(np.ascontiguousarray(w)).cuda()
        dwm.dwm_filter_transform(self.plan, self.w.data_ptr(), self.Ugw.data_ptr(), self.stream())

    def forward(self, x):
        self.x = torch.from_numpy(np.ascontiguousarray(x)).cuda()
        dwm.dwm_conv_forward(self.plan, self.x.data_ptr(), self.Ugw.data_ptr(), self.y.data_ptr(), self.stream())
        torch.cuda.synchronize()
        return self.y.cpu().numpy()

    def classes(self):
        return [dwm.dwm_plan_class(self.plan, i) for i in range(self.info.n_classes)]

    def parts(self):
        return [dwm.dwm_plan_part(self.plan, i) for i in range(self.info.n_parts)]

    def close(self):
        torch.cuda.synchronize()
        dwm.dwm_plan_destroy(self.plan)


def conv(x, w, stride, pad, variants=None):
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    r = Runner(N, C, H, W, K, R, S, stride, pad, variants)
    try:
        r.set_filter(w)
        return r.forward(x)
    finally:
        r.close()
