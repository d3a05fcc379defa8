// HIP kernels of libdwm for gfx950 (MI355X): filter transform and input transform, the
// "Transformation" step of the paper's Sec. 4.1 list on the kernel and on the input side
// (the input side includes the "Splitting" of the input into per-part, per-phase views).
// Winograd matrices are those of Sec. 3.2 for F(2,3) and the 0/1-entry three- and
// two-multiplication forms for 2-tap and 1-tap pieces.
#include <hip/hip_runtime.h>

#include "plan.hpp"
#include "xform.hpp"

namespace dwm {

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
            const int ih = P.s * (2 * ty + hp.j + i) + hp.p - P.Ph;
#pragma unroll
            for (int j = 0; j < TW_; ++j) {
                const int iw = P.s * (2 * tx + wp.j + j) + wp.p - P.Pw;
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
// Input transform, LDS-staged form.
//
// A workgroup owns one 64-tile block of V (lane = tile) and `cg` input channels.  Each of
// its four waves stages the input rows that the block's tiles touch, for ITS channels
// (c = c0 + wave, c0 + wave + 4, ...), once, with coalesced loads: zero padding is written
// explicitly and columns are de-interleaved modulo 2*stride, so that the same patch element
// of adjacent tiles sits in adjacent LDS words.  The wave then walks every part of every
// class for those channels: a patch element is one LDS read at (lane's tile base) + (an
// offset that is the same for the whole wave).  x is read from HBM about once and every
// load instruction is fully used; the global-memory gathers of the other form (one 4-byte
// load per patch element, lanes 2*stride floats apart) are gone.  Waves never wait for each
// other: a wave reads only what it staged itself.
// The 64 tiles of a block span a few tile rows, possibly of several images: the staged rows
// are the union per image ("segments"), stored one after the other.
// ---------------------------------------------------------------------------------
template <int LH, int LW>
__device__ __forceinline__ void lds_class_rows(const DevPlan& P, const InLdsArgs& A, const DevClass& q,
                                               const float* __restrict__ xl, float* __restrict__ vb, int c0,
                                               int cn, int wave, bool valid)
{
    constexpr int TH_ = LH + 1, TW_ = LW + 1;
    const size_t plane = (size_t)q.Lpad * 64;
    for (int a = 0; a < q.hn; ++a)
        for (int b = 0; b < q.wn; ++b) {
            int ro[TH_], co[TW_];
#pragma unroll
            for (int i = 0; i < TH_; ++i) ro[i] = A.roff[q.h0 + a][i];
#pragma unroll
            for (int j = 0; j < TW_; ++j) co[j] = A.coff[q.w0 + b][j];
            const int lbase = (a * q.wn + b) * P.C + c0;
            for (int cl = wave; cl < cn; cl += 4) {
                const float* xc = xl + cl * A.chan_floats;
                float d[TH_][TW_];
#pragma unroll
                for (int i = 0; i < TH_; ++i)
#pragma unroll
                    for (int j = 0; j < TW_; ++j) d[i][j] = xc[ro[i] + co[j]];
                float* vp = vb + (size_t)(q.v_row0 + lbase + cl) * 64;
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
                    if (valid) {
#pragma unroll
                        for (int j = 0; j < TW_; ++j) vp[(size_t)(i * TW_ + j) * plane] = o[j];
                    }
                }
            }
        }
}

__global__ __launch_bounds__(256) void input_transform_lds_kernel(DevPlan P, InLdsArgs A,
                                                                  const float* __restrict__ x,
                                                                  float* __restrict__ V, int* __restrict__ counters,
                                                                  int n_counters, int chan_fast, int write_pad_rows)
{
    extern __shared__ __attribute__((aligned(16))) float xs[];  // [cg][max_rows][nphase][lwp]
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < n_counters; i += blockDim.x) counters[i] = 0;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nbt = P.Tpad / 64;
    const int b = blockIdx.x;
    const int bt = chan_fast ? b / A.ncg : b % nbt, bc = chan_fast ? b % A.ncg : b / nbt;
    const int c0 = bc * A.cg, cn = min(A.cg, P.C - c0);
    const int t0 = bt * 64;
    if (t0 >= P.T) return;  // a block of padding only (Tpad is rounded up to 256)
    const int t1 = min(t0 + 63, P.T - 1);
    const int s2 = 2 * P.s;
    const int g0 = A.div_tw.div(t0), g1 = A.div_tw.div(t1);
    const int n0 = A.div_th.div(g0), n1 = A.div_th.div(g1);
    const int ty_a0 = g0 - n0 * P.TH, ty_b1 = g1 - n1 * P.TH;
    const int rows0 = s2 * ((n1 == n0 ? ty_b1 : P.TH - 1) - ty_a0) + A.foot_h;

    // ---- 1. this wave stages its channels: lanes along a row, rows in batches of up to
    // kInLdsBatch loads, segment by segment.  Rows above or below the image are written as
    // zeros; columns left or right of it are loaded from a clamped (legal) address and
    // replaced by zero on the way to LDS.
    for (int cl = wave; cl < cn; cl += 4)
        stage_channels<float, 1>(P, A, x, xs + cl * A.chan_floats, c0 + cl, 4, n0, n1, ty_a0, ty_b1, lane);

    // ---- 2. every part of every class for those channels ----
    const int t = t0 + lane;
    const bool valid = t < P.T;
    int lane_base = 0;
    if (valid) {
        const int g = A.div_tw.div(t), tx = t - g * P.TW;
        const int n = A.div_th.div(g), ty = g - n * P.TH;
        const int base_row = n == n0 ? s2 * (ty - ty_a0) : rows0 + (n - n0 - 1) * A.rows_full + s2 * ty;
        lane_base = base_row * A.row_floats + tx;
    }
    const float* xl = xs + lane_base;
    float* vb = V + (size_t)bt * P.vblock_rows * 64 + lane;
    for (int qi = 0; qi < P.ncls; ++qi) {
        const DevClass q = P.cls[qi];
        switch (q.lh * 4 + q.lw) {
            case 3 * 4 + 3: lds_class_rows<3, 3>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            case 3 * 4 + 2: lds_class_rows<3, 2>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            case 3 * 4 + 1: lds_class_rows<3, 1>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            case 2 * 4 + 3: lds_class_rows<2, 3>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            case 2 * 4 + 2: lds_class_rows<2, 2>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            case 2 * 4 + 1: lds_class_rows<2, 1>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            case 1 * 4 + 3: lds_class_rows<1, 3>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            case 1 * 4 + 2: lds_class_rows<1, 2>(P, A, q, xl, vb, c0, cn, wave, valid); break;
            default: lds_class_rows<1, 1>(P, A, q, xl, vb, c0, cn, wave, valid); break;
        }
        // rows past the class's reduction length are zeros (the contraction multiplies them)
        if (bc == 0 && valid && write_pad_rows) {
            const int planes = (q.lh + 1) * (q.lw + 1);
            for (int l = q.L + wave; l < q.Lpad; l += 4)
                for (int pl = 0; pl < planes; ++pl) vb[((size_t)q.v_row0 + (size_t)pl * q.Lpad + l) * 64] = 0.f;
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

dwm_status_t launch_filter_transform(const dwm_plan& p, const float* w, float* U, void* stream)
{
    dim3 grid((p.d.rows_total + 255) / 256, p.d.Kpad), block(256);
    hipLaunchKernelGGL(filter_transform_kernel, grid, block, 0, (hipStream_t)stream, p.d, w, U);
    return check_launch();
}

dwm_status_t launch_input_transform(const dwm_plan& p, const float* x, float* V, void* stream)
{
    const DevPlan& d = p.d;
    const int nb = d.Tpad / 64, nr = d.rows_total / 16;
    dim3 block(256);
    // variants: 0/1 = gather form (blocks-fast / rows-fast), 2/3 = LDS-staged form (channel groups
    // fastest / blocks fastest); planner's choice: LDS-staged where it applies
    int variant = p.variant_input;
    if (variant < 0) variant = p.inlds_ok ? 2 : ((size_t)d.N * d.C * d.H * d.W * sizeof(float) > ((size_t)64 << 20));
    if (variant >= 2) {
        if (!p.inlds_ok) return DWM_ERR_INVALID_ARG;
        const InLdsArgs& a = p.inlds;
        auto kernel = input_transform_lds_kernel;
        if (a.lds_bytes > 64 * 1024) {
            static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (attr != hipSuccess) return DWM_ERR_HIP;
        }
        hipLaunchKernelGGL(kernel, dim3((unsigned)(nb * a.ncg)), block, a.lds_bytes, (hipStream_t)stream, d, a, x, V,
                           p.sk_counters(V), p.geo.n_sk_tiles, variant == 2, p.skip_pad_rows ? 0 : 1);
        return check_launch();
    }
    int rows_fast = variant;
    if ((rows_fast ? nb : nr) > 65535) rows_fast = !rows_fast;
    if ((rows_fast ? nb : nr) > 65535) return DWM_ERR_UNSUPPORTED;
    dim3 grid(rows_fast ? nr : nb, rows_fast ? nb : nr);
    hipLaunchKernelGGL(input_transform_kernel, grid, block, 0, (hipStream_t)stream, d, x, V, p.sk_counters(V),
                       p.geo.n_sk_tiles, rows_fast);
    return check_launch();
}

}  // namespace dwm
