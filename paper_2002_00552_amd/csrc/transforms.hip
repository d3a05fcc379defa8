// HIP kernels of libdwm for gfx950 (MI355X): filter transform and input transform, the
// "Transformation" step of the paper's Sec. 4.1 list on the kernel and on the input side
// (the input side includes the "Splitting" of the input into per-part, per-phase views).
// Winograd matrices are those of Sec. 3.2 for F(2,3) and the 0/1-entry three- and
// two-multiplication forms for 2-tap and 1-tap pieces.
#include <hip/hip_runtime.h>

#include "plan.hpp"

namespace dwm {

// ---------------------------------------------------------------------------------
// 1-D transforms, one row at a time
// ---------------------------------------------------------------------------------

// (G_l v)[i] for a piece of length l (v has l valid entries).
__device__ __forceinline__ float g_row(int l, int i, float v0, float v1, float v2)
{
    if (l == 3) {
        switch (i) {
            case 0: return v0;
            case 1: return 0.5f * (v0 + v1 + v2);
            case 2: return 0.5f * (v0 - v1 + v2);
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

// ---------------------------------------------------------------------------------
// Filter transform: U = G_lh g G_lw^T for every part (Sec. 4.1 "Transformation")
// One thread per (row of the flattened (class, l) space, k); writes all planes of its
// class, zeros in the padding.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void filter_transform_kernel(DevPlan P, const float* __restrict__ w,
                                                               float* __restrict__ U)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (row >= P.rows_total) return;
    const int qi = find_class(P, row);
    const DevClass q = P.cls[qi];
    const int l = row - q.row0;
    const int th = q.lh + 1, tw = q.lw + 1;

    float u[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) u[i][j] = 0.f;

    if (l < q.L && k < P.K) {
        const int slot = l / P.C, c = l - slot * P.C;
        const int a = slot / q.wn, b = slot - a * q.wn;
        const DevPiece hp = P.ph[q.h0 + a], wp = P.pw[q.w0 + b];
        float g[3][3];
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                float v = 0.f;
                if (i < q.lh && j < q.lw) {
                    const int r = P.s * (hp.j + i) + hp.p, s2 = P.s * (wp.j + j) + wp.p;
                    v = w[(((size_t)k * P.C + c) * P.R + r) * P.S + s2];
                }
                g[i][j] = v;
            }
        float t[4][3];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j) t[i][j] = (i < th) ? g_row(q.lh, i, g[0][j], g[1][j], g[2][j]) : 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) u[i][j] = (i < th && j < tw) ? g_row(q.lw, j, t[i][0], t[i][1], t[i][2]) : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i < th && j < tw) {
                U[(size_t)q.u_off + ((size_t)(i * tw + j) * P.Kpad + k) * q.Lpad + l] = u[i][j];
                if (P.has_ut && l < q.Lt)
                    U[(size_t)q.ut_off + ((size_t)(i * tw + j) * q.Lt + l) * P.Kpad + k] = u[i][j];
            }
}

// ---------------------------------------------------------------------------------
// Input transform: V = B^T d B for every part (Sec. 4.1 "Splitting" of the input and
// "Transformation").
//
// A thread owns one tile t and FOUR consecutive rows l of the flattened (class, l) space
// (four channels of one part, as a rule).  For each row it gathers the part's
// (lh+1)x(lw+1) patch d[a][b] = xp[s(2ty+jh+a)+ph][s(2tx+jw+b)+pw] (phase p of the padded
// input, eq. 14 generalised to any stride) straight from global memory -- L1/L2 absorb the
// re-reads of overlapping patches; all four rows' loads are issued before the first use so
// that enough bytes are in flight -- applies the transform and writes one value per plane.
// V is blocked by 64 tiles: a wave's store is one 256-byte row, a workgroup (64 tiles x 16
// rows) writes 4 KB contiguous per plane.
// ---------------------------------------------------------------------------------
template <int LH, int LW>
__device__ __forceinline__ void input_rows4(const DevPlan& P, const DevClass& q, const float* __restrict__ x,
                                            float* __restrict__ V, int l0, int t)
{
    constexpr int TH_ = LH + 1, TW_ = LW + 1;
    float d[4][TH_][TW_];
    const bool t_ok = t < P.T;
    const int tiles = P.TH * P.TW;
    const int n = t / tiles, rem = t - n * tiles;
    const int ty = rem / P.TW, tx = rem - ty * P.TW;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int l = l0 + r;
        const bool ok = l < q.L && t_ok;
        const int slot = l / P.C, c = l - slot * P.C;
        const int a = slot / q.wn, b = slot - a * q.wn;
        const DevPiece hp = P.ph[q.h0 + (ok ? a : 0)], wp = P.pw[q.w0 + (ok ? b : 0)];
        const float* xc = x + ((size_t)n * P.C + c) * P.H * P.W;
#pragma unroll
        for (int i = 0; i < TH_; ++i) {
            const int ih = P.s * (2 * ty + hp.j + i) + hp.p - P.P;
#pragma unroll
            for (int j = 0; j < TW_; ++j) {
                const int iw = P.s * (2 * tx + wp.j + j) + wp.p - P.P;
                d[r][i][j] = (ok && ih >= 0 && ih < P.H && iw >= 0 && iw < P.W) ? xc[(size_t)ih * P.W + iw] : 0.f;
            }
        }
    }
    if (!t_ok) return;  // columns past the last tile are never read back into y
    float* vp = V + (size_t)(t >> 6) * P.vblock_rows * 64 + (size_t)(q.v_row0 + l0) * 64 + (t & 63);
    const size_t plane = (size_t)q.Lpad * 64;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        // columns first (B^T d), then rows ((B^T d) B)
        float tmp[4][4];
#pragma unroll
        for (int j = 0; j < TW_; ++j) {
            float col[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
#pragma unroll
            for (int i = 0; i < TH_; ++i) col[i] = d[r][i][j];
            bt_apply<LH>(col, o);
#pragma unroll
            for (int i = 0; i < TH_; ++i) tmp[i][j] = o[i];
        }
#pragma unroll
        for (int i = 0; i < TH_; ++i) {
            float rowv[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
#pragma unroll
            for (int j = 0; j < TW_; ++j) rowv[j] = tmp[i][j];
            bt_apply<LW>(rowv, o);
#pragma unroll
            for (int j = 0; j < TW_; ++j) vp[(size_t)(i * TW_ + j) * plane + r * 64] = o[j];
        }
    }
}

__global__ __launch_bounds__(256) void input_transform_kernel(DevPlan P, const float* __restrict__ x,
                                                              float* __restrict__ V, int* __restrict__ counters,
                                                              int n_counters, int rows_fast)
{
    // The contraction that follows counts partial-tile arrivals in `counters`; they start at zero.
    if (blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = threadIdx.x; i < n_counters; i += blockDim.x) counters[i] = 0;

    // Workgroup order.  rows_fast: consecutive workgroups take consecutive row groups of the SAME
    // 64-tile block, so every part and channel of those tiles is in flight together and x is
    // fetched from HBM once (it matters when x outgrows the L2).  Otherwise consecutive
    // workgroups take consecutive blocks of the same rows (measured faster while x stays cached).
    const int bt = rows_fast ? blockIdx.y : blockIdx.x, br = rows_fast ? blockIdx.x : blockIdx.y;
    const int t = bt * 64 + (threadIdx.x & 63);          // < Tpad by construction of the grid
    const int row = br * 16 + (threadIdx.x >> 6) * 4;    // 4 rows, never across a class (Lpad % 16 == 0)
    const int qi = find_class(P, row);
    const DevClass q = P.cls[qi];
    const int l0 = row - q.row0;
    switch (q.lh * 4 + q.lw) {
        case 3 * 4 + 3: input_rows4<3, 3>(P, q, x, V, l0, t); break;
        case 3 * 4 + 2: input_rows4<3, 2>(P, q, x, V, l0, t); break;
        case 3 * 4 + 1: input_rows4<3, 1>(P, q, x, V, l0, t); break;
        case 2 * 4 + 3: input_rows4<2, 3>(P, q, x, V, l0, t); break;
        case 2 * 4 + 2: input_rows4<2, 2>(P, q, x, V, l0, t); break;
        case 2 * 4 + 1: input_rows4<2, 1>(P, q, x, V, l0, t); break;
        case 1 * 4 + 3: input_rows4<1, 3>(P, q, x, V, l0, t); break;
        case 1 * 4 + 2: input_rows4<1, 2>(P, q, x, V, l0, t); break;
        default: input_rows4<1, 1>(P, q, x, V, l0, t); break;
    }
}

// ---------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------
static dwm_status_t check_launch()
{
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

__global__ __launch_bounds__(256) void zero_fill_kernel(float* __restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}

dwm_status_t launch_filter_transform(const dwm_plan& p, const float* w, float* U, void* stream)
{
    dim3 grid((p.d.rows_total + 255) / 256, p.d.Kpad), block(256);
    hipLaunchKernelGGL(filter_transform_kernel, grid, block, 0, (hipStream_t)stream, p.d, w, U);
    if (p.d.has_ut) {  // the slack rows after the transposed copy (read, never used)
        const size_t slack = (size_t)32 * p.d.Kpad;
        hipLaunchKernelGGL(zero_fill_kernel, dim3(32), block, 0, (hipStream_t)stream,
                           U + p.filter_floats - slack, slack);
    }
    return check_launch();
}

dwm_status_t launch_input_transform(const dwm_plan& p, const float* x, float* V, void* stream)
{
    const DevPlan& d = p.d;
    const int nb = d.Tpad / 64, nr = d.rows_total / 16;
    int rows_fast = (size_t)d.N * d.C * d.H * d.W * sizeof(float) > ((size_t)64 << 20);
    if (p.variant_input == 0 || p.variant_input == 1) rows_fast = p.variant_input;
    if ((rows_fast ? nb : nr) > 65535) rows_fast = !rows_fast;
    if ((rows_fast ? nb : nr) > 65535) return DWM_ERR_UNSUPPORTED;
    dim3 grid(rows_fast ? nr : nb, rows_fast ? nb : nr), block(256);
    hipLaunchKernelGGL(input_transform_kernel, grid, block, 0, (hipStream_t)stream, d, x, V, p.sk_counters(),
                       p.geo.n_sk_tiles, rows_fast);
    return check_launch();
}

}  // namespace dwm
