// 1-D Winograd transforms of the staged path, one row at a time, shared by the single- and the
// half-precision kernels: F(2,3) as printed in the paper's Sec. 3.2, and the 0/1-entry three- and
// two-multiplication forms for 2-tap and 1-tap pieces.
#pragma once
#include <hip/hip_runtime.h>

#include "plan.hpp"

namespace dwm {

// (G_l v)[i] for a piece of length l (v has l valid entries).
template <typename F>
__device__ __forceinline__ F g_row(int l, int i, F v0, F v1, F v2)
{
    if (l == 3) {
        switch (i) {
            case 0: return v0;
            case 1: return F(0.5) * (v0 + v1 + v2);
            case 2: return F(0.5) * (v0 - v1 + v2);
            default: return v2;
        }
    }
    if (l == 2) return i == 0 ? v0 : i == 1 ? v0 + v1 : v1;
    return v0;
}

// (B_l^T d)[i] for a piece of length l (d has l+1 valid entries).
template <int L>
__device__ __forceinline__ void bt_apply(const float d[4], float out[4])
{
    if (L == 3) {
        out[0] = d[0] - d[2];
        out[1] = d[1] + d[2];
        out[2] = d[2] - d[1];
        out[3] = d[1] - d[3];
    } else if (L == 2) {
        out[0] = d[0] - d[1];
        out[1] = d[1];
        out[2] = d[2] - d[1];
    } else {
        out[0] = d[0];
        out[1] = d[1];
    }
}

__device__ __forceinline__ int find_class(const DevPlan& P, int row)
{
    int q = 0;
    while (q + 1 < P.ncls && row >= P.cls[q + 1].row0) ++q;
    return q;
}

}  // namespace dwm
