// HIP kernels of libdwm for gfx950 (MI355X): filter transform and input transform, the
// "Transformation" step of the paper's Sec. 4.1 list on the kernel and on the input side
// (the input side includes the "Splitting" of the input into per-part, per-phase views).
// Winograd matrices are those of Sec. 3.2 for F(2,3) and the 0/1-entry three- and
// two-multiplication forms for 2-tap and 1-tap pieces.
#include <hip/hip_runtime.h>

#include <algorithm>

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
// Input transform, gather form: one thread per (row of the (class, l) space, tile t).
// Reads the part's (lh+1)x(lw+1) patch d[a][b] = xp[s(2ty+jh+a)+ph][s(2tx+jw+b)+pw]
// (phase p of the padded input, Sec. 4.1 eq. 14 generalised to any stride), applies
// V = B^T d B and writes one value per plane, coalesced along t.
// ---------------------------------------------------------------------------------
template <int LH, int LW>
__device__ __forceinline__ void input_tile(const DevPlan& P, const DevClass& q, const float* __restrict__ x,
                                           float* __restrict__ V, int l, int t)
{
    constexpr int TH_ = LH + 1, TW_ = LW + 1;
    float v[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) v[i][j] = 0.f;

    if (l < q.L && t < P.T) {
        const int slot = l / P.C, c = l - slot * P.C;
        const int a = slot / q.wn, b = slot - a * q.wn;
        const DevPiece hp = P.ph[q.h0 + a], wp = P.pw[q.w0 + b];
        const int tiles = P.TH * P.TW;
        const int n = t / tiles, rem = t - n * tiles;
        const int ty = rem / P.TW, tx = rem - ty * P.TW;
        const float* xc = x + ((size_t)n * P.C + c) * P.H * P.W;
        float d[4][4];
#pragma unroll
        for (int i = 0; i < TH_; ++i) {
            const int ih = P.s * (2 * ty + hp.j + i) + hp.p - P.P;
#pragma unroll
            for (int j = 0; j < TW_; ++j) {
                const int iw = P.s * (2 * tx + wp.j + j) + wp.p - P.P;
                d[i][j] = (ih >= 0 && ih < P.H && iw >= 0 && iw < P.W) ? xc[(size_t)ih * P.W + iw] : 0.f;
            }
        }
        // columns first (B^T d), then rows ((B^T d) B)
        float tmp[4][4];
#pragma unroll
        for (int j = 0; j < TW_; ++j) {
            float col[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
#pragma unroll
            for (int i = 0; i < TH_; ++i) col[i] = d[i][j];
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
            for (int j = 0; j < TW_; ++j) v[i][j] = o[j];
        }
    }
#pragma unroll
    for (int i = 0; i < TH_; ++i)
#pragma unroll
        for (int j = 0; j < TW_; ++j)
            V[(size_t)q.v_off + ((size_t)(i * TW_ + j) * q.Lpad + l) * P.Tpad + t] = v[i][j];
}

__global__ __launch_bounds__(256) void input_transform_gather_kernel(DevPlan P, const float* __restrict__ x,
                                                                     float* __restrict__ V,
                                                                     int* __restrict__ counters, int n_counters)
{
    // The contraction that follows counts partial-tile arrivals in `counters`; they start at zero.
    if (blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = threadIdx.x; i < n_counters; i += blockDim.x) counters[i] = 0;

    const int t = blockIdx.x * blockDim.x + threadIdx.x;  // < Tpad by construction of the grid
    const int row = blockIdx.y;
    const int qi = find_class(P, row);
    const DevClass q = P.cls[qi];
    const int l = row - q.row0;
    switch (q.lh * 4 + q.lw) {
        case 3 * 4 + 3: input_tile<3, 3>(P, q, x, V, l, t); break;
        case 3 * 4 + 2: input_tile<3, 2>(P, q, x, V, l, t); break;
        case 3 * 4 + 1: input_tile<3, 1>(P, q, x, V, l, t); break;
        case 2 * 4 + 3: input_tile<2, 3>(P, q, x, V, l, t); break;
        case 2 * 4 + 2: input_tile<2, 2>(P, q, x, V, l, t); break;
        case 2 * 4 + 1: input_tile<2, 1>(P, q, x, V, l, t); break;
        case 1 * 4 + 3: input_tile<1, 3>(P, q, x, V, l, t); break;
        case 1 * 4 + 2: input_tile<1, 2>(P, q, x, V, l, t); break;
        default: input_tile<1, 1>(P, q, x, V, l, t); break;
    }
}

// ---------------------------------------------------------------------------------
// Input transform, LDS-staged form (variant 0; measured no faster than the gather form).
//
// A workgroup owns one image n, one channel c and a band of BT tile rows.  It reads the
// input rows the band needs ONCE, coalesced, into LDS -- zero padding written explicitly,
// columns de-interleaved by their residue modulo 2*stride so that the patches of
// neighbouring tiles, which sit 2*stride columns apart (a polyphase view at twice the
// stride), are contiguous in LDS -- and then every thread takes (part, tile) items:
// gathers the part's patch from LDS, applies V = B^T d B and writes one value per plane.
// Lanes of a wave hold consecutive tiles, so every store is a contiguous run along t.
// The workgroups with c == C write the zero rows that pad each class's reduction length.
// ---------------------------------------------------------------------------------
struct InputArgs {
    int BT, nbands;    // tile rows per band, bands per image
    int nphase;        // 2*stride
    int lwp;           // LDS floats per (row, phase)
    int lw_in;         // padded input columns staged per row
    int max_oh;        // largest row offset s*(j+l)+p over the h-pieces
    int tile_row_step; // LDS floats between the patches of vertically adjacent tiles
    FastDiv div_tw, div_nphase;
    // LDS offset of patch row a of h-piece i / patch column b of w-piece i
    int roff[kMaxPieces][4], coff[kMaxPieces][4];
};

template <int LH, int LW>
__device__ __forceinline__ void lds_tile(const float* __restrict__ xs, const int* __restrict__ roff,
                                         const int* __restrict__ coff, float* __restrict__ vp, size_t plane)
{
    constexpr int TH_ = LH + 1, TW_ = LW + 1;
    float d[4][4];
#pragma unroll
    for (int i = 0; i < TH_; ++i)
#pragma unroll
        for (int j = 0; j < TW_; ++j) d[i][j] = xs[roff[i] + coff[j]];
    float tmp[4][4], v[4][4];
#pragma unroll
    for (int j = 0; j < TW_; ++j) {
        float col[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
#pragma unroll
        for (int i = 0; i < TH_; ++i) col[i] = d[i][j];
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
        for (int j = 0; j < TW_; ++j) v[i][j] = o[j];
    }
#pragma unroll
    for (int i = 0; i < TH_; ++i)
#pragma unroll
        for (int j = 0; j < TW_; ++j) vp[(size_t)(i * TW_ + j) * plane] = v[i][j];
}

__global__ __launch_bounds__(256) void input_transform_lds_kernel(DevPlan P, InputArgs a,
                                                                  const float* __restrict__ x, float* __restrict__ V,
                                                                  int* __restrict__ counters, int n_counters)
{
    extern __shared__ float xs[];  // [row][phase][lwp]
    const int tid = threadIdx.x;
    // The contraction that follows counts partial-tile arrivals in `counters`; they start at zero.
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
        for (int i = tid; i < n_counters; i += 256) counters[i] = 0;

    const int band = blockIdx.x, c = blockIdx.y, n = blockIdx.z;
    const int ty0 = band * a.BT;
    const int bt = (P.TH - ty0 < a.BT) ? P.TH - ty0 : a.BT;
    const int ntb = bt * P.TW;
    const size_t t0 = ((size_t)n * P.TH + ty0) * P.TW;

    if (c == P.C) {  // zero rows l in [L, Lpad) of every plane, for this band's tiles
        for (int qi = 0; qi < P.ncls; ++qi) {
            const DevClass q = P.cls[qi];
            const int planes = (q.lh + 1) * (q.lw + 1);
            for (int pl = 0; pl < planes; ++pl)
                for (int l = q.L; l < q.Lpad; ++l) {
                    float* vp = V + (size_t)q.v_off + ((size_t)pl * q.Lpad + l) * P.Tpad + t0;
                    for (int i = tid; i < ntb; i += 256) vp[i] = 0.f;
                }
        }
        return;
    }

    // stage the band's input rows (padded coordinates: row 0 of the band is padded row 2*ty0*s);
    // a wave takes a row, its lanes consecutive columns
    const int nrows = 2 * P.s * (bt - 1) + a.max_oh + 1;
    const int prow0 = 2 * ty0 * P.s;
    const float* xc = x + ((size_t)n * P.C + c) * P.H * P.W;
    for (int r = tid >> 6; r < nrows; r += 4) {
        const int ih = prow0 + r - P.P;
        const bool row_ok = ih >= 0 && ih < P.H;
        const float* xr = xc + (size_t)ih * P.W - P.P;
        float* xsr = xs + r * a.nphase * a.lwp;
        for (int col = tid & 63; col < a.lw_in; col += 64) {
            const int iw = col - P.P;
            const float v = (row_ok && iw >= 0 && iw < P.W) ? xr[col] : 0.f;
            const int idx = a.div_nphase.div(col);
            xsr[(col - idx * a.nphase) * a.lwp + idx] = v;
        }
    }
    __syncthreads();

    // a thread takes a tile of the band and walks all parts; everything that depends on the
    // part is the same for all threads (scalar registers)
    for (int i = tid; i < ntb; i += 256) {
        const int ty = a.div_tw.div(i), tx = i - ty * P.TW;
        const float* xt = xs + ty * a.tile_row_step + tx;
        float* vt = V + t0 + i;
        for (int qi = 0; qi < P.ncls; ++qi) {
            const DevClass q = P.cls[qi];
            const size_t plane = (size_t)q.Lpad * P.Tpad;
            for (int ah = 0; ah < q.hn; ++ah)
                for (int bw = 0; bw < q.wn; ++bw) {
                    const int l = (ah * q.wn + bw) * P.C + c;
                    float* vp = vt + (size_t)q.v_off + (size_t)l * P.Tpad;
                    const int* ro = a.roff[q.h0 + ah];
                    const int* co = a.coff[q.w0 + bw];
                    switch (q.lh * 4 + q.lw) {
                        case 3 * 4 + 3: lds_tile<3, 3>(xt, ro, co, vp, plane); break;
                        case 3 * 4 + 2: lds_tile<3, 2>(xt, ro, co, vp, plane); break;
                        case 3 * 4 + 1: lds_tile<3, 1>(xt, ro, co, vp, plane); break;
                        case 2 * 4 + 3: lds_tile<2, 3>(xt, ro, co, vp, plane); break;
                        case 2 * 4 + 2: lds_tile<2, 2>(xt, ro, co, vp, plane); break;
                        case 2 * 4 + 1: lds_tile<2, 1>(xt, ro, co, vp, plane); break;
                        case 1 * 4 + 3: lds_tile<1, 3>(xt, ro, co, vp, plane); break;
                        case 1 * 4 + 2: lds_tile<1, 2>(xt, ro, co, vp, plane); break;
                        default: lds_tile<1, 1>(xt, ro, co, vp, plane); break;
                    }
                }
        }
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
    if (p.variant_input != 0) {  // gather form (the default): no LDS, one thread per (row, tile)
        if (d.rows_total > 65535) return DWM_ERR_UNSUPPORTED;
        dim3 grid(d.Tpad / 256, d.rows_total), block(256);
        hipLaunchKernelGGL(input_transform_gather_kernel, grid, block, 0, (hipStream_t)stream, d, x, V,
                           p.sk_counters(), p.geo.n_sk_tiles);
        return check_launch();
    }
    // LDS-staged form: pick the band height so that a band's rows fit in 48 KB of LDS
    InputArgs a;
    int max_oh = 0, max_ow = 0;
    for (int i = 0; i < d.nh; ++i) max_oh = std::max(max_oh, d.s * (d.ph[i].j + d.ph[i].l) + d.ph[i].p);
    for (int i = 0; i < d.nw; ++i) max_ow = std::max(max_ow, d.s * (d.pw[i].j + d.pw[i].l) + d.pw[i].p);
    a.nphase = 2 * d.s;
    a.max_oh = max_oh;
    a.lw_in = 2 * d.s * (d.TW - 1) + max_ow + 1;
    a.lwp = (a.lw_in + a.nphase - 1) / a.nphase;
    a.lwp |= 1;  // odd: the staging writes of one row spread over the banks
    const long long row_floats = (long long)a.nphase * a.lwp;
    const long long budget = 48 * 1024 / 4;
    long long bt = (budget / row_floats - max_oh - 1) / (2 * d.s) + 1;
    if (bt < 1) return DWM_ERR_UNSUPPORTED;  // one tile row of this width does not fit in LDS
    if (bt > d.TH) bt = d.TH;
    a.nbands = (int)((d.TH + bt - 1) / bt);
    a.BT = (d.TH + a.nbands - 1) / a.nbands;
    const int rows_max = 2 * d.s * (a.BT - 1) + max_oh + 1;
    a.tile_row_step = 2 * d.s * (int)row_floats;
    a.div_tw.init((unsigned)d.TW);
    a.div_nphase.init((unsigned)a.nphase);
    for (int i = 0; i < kMaxPieces; ++i)
        for (int k = 0; k < 4; ++k) {
            const int oh = i < d.nh ? d.s * (d.ph[i].j + k) + d.ph[i].p : 0;
            const int ow = i < d.nw ? d.s * (d.pw[i].j + k) + d.pw[i].p : 0;
            a.roff[i][k] = oh * (int)row_floats;
            a.coff[i][k] = (ow % a.nphase) * a.lwp + ow / a.nphase;
        }
    if (d.C + 1 > 65535 || d.N > 65535) return DWM_ERR_UNSUPPORTED;
    const size_t lds = (size_t)rows_max * row_floats * sizeof(float);
    bool any_pad = false;
    for (int i = 0; i < d.ncls; ++i) any_pad |= d.cls[i].Lpad != d.cls[i].L;
    dim3 grid(a.nbands, d.C + (any_pad ? 1 : 0), d.N), block(256);
    hipLaunchKernelGGL(input_transform_lds_kernel, grid, block, lds, (hipStream_t)stream, d, a, x, V,
                       p.sk_counters(), p.geo.n_sk_tiles);
    return check_launch();
}

}  // namespace dwm
