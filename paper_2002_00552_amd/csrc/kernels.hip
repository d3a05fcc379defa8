// HIP kernels of libdwm for gfx950 (MI355X): filter transform, input transform, and the
// per-plane MFMA contraction with the output transform and aggregation fused into its
// epilogue.  Steps follow the paper's Sec. 4.1 list (splitting, transformation,
// calculation, detransformation, aggregation); Winograd matrices are those of Sec. 3.2
// for F(2,3) and the 0/1-entry three- and two-multiplication forms for 2-tap and 1-tap
// pieces.
#include <hip/hip_runtime.h>

#include "plan.hpp"

namespace dwm {

typedef float floatx16 __attribute__((ext_vector_type(16)));

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
            if (i < th && j < tw)
                U[(size_t)q.u_off + ((size_t)(i * tw + j) * P.Kpad + k) * q.Lpad + l] = u[i][j];
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
                                                                     float* __restrict__ V)
{
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
// Contraction + output transform + aggregation (Sec. 4.1 "Calculation",
// "Detransformation", "Aggregation").
//
// For each plane p = (class, fh, fw):  M_p[k][t] = sum_l U_p[k][l] * V_p[l][t]  -- the
// element-wise product summed over channels, and over the parts of the class because
// A^T(.)A is linear -- a GEMM on fp32 MFMA.  Since the output transform is linear too,
// Y[k][t][a][b] = sum_p AT_lh[a][fh] * AT_lw[b][fw] * M_p[k][t] with coefficients in
// {0,+1,-1}: a workgroup owns a (K tile, T tile), walks the planes one after the other,
// keeps ONE MFMA accumulator and folds it into four running 2x2 outputs when the plane's
// reduction ends.  M never exists in memory; y is written once.
//
// Workgroup = 4 waves as 2 (K) x 2 (T); a wave owns (32*WM) x (32*WN) of the tile and
// uses v_mfma_f32_32x32x2_f32.  U and V chunks of LC reduction steps are staged through
// double-buffered LDS.  Within a group of 8 reduction steps the MFMA with index s takes
// steps {s, 4+s} as its two k-slots, so a lane's A operands for four MFMAs are one
// 16-byte LDS read.
// ---------------------------------------------------------------------------------
struct ContractArgs {
    int K, T, Kpad, Tpad;
    int OH, OW, TH, TW;
    int nkt, ntt;
};

template <int WM, int WN, int LC>
__global__ __launch_bounds__(256, 2) void contract_output_kernel(ContractArgs A, PlaneTable PT,
                                                                 const float* __restrict__ U,
                                                                 const float* __restrict__ V,
                                                                 float* __restrict__ y)
{
    constexpr int KT = 64 * WM, TT = 64 * WN;
    constexpr int AS = LC + 4;  // LDS row stride of the U tile (floats)
    constexpr int BS = TT + 8;  // LDS row stride of the V tile (floats)
    constexpr int A_C4 = LC / 4;          // float4 per U row
    constexpr int A_ROWS = 256 / A_C4;    // U rows per pass
    constexpr int A_PASS = KT / A_ROWS;
    constexpr int B_C4 = TT / 4;          // float4 per V row
    constexpr int B_ROWS = 256 / B_C4;    // V rows per pass
    constexpr int B_PASS = LC / B_ROWS;
    static_assert(A_PASS >= 1 && B_PASS >= 1 && KT % A_ROWS == 0 && LC % B_ROWS == 0, "tile/thread mismatch");

    __shared__ __attribute__((aligned(16))) float As[2][KT * AS];
    __shared__ __attribute__((aligned(16))) float Bs[2][LC * BS];

    // XCD-aware tile order: workgroups are dealt round-robin to the 8 XCDs, so the
    // K tiles of one T tile are given consecutive slots on ONE XCD and share its L2.
    const int b = blockIdx.x;
    const int xcd = b & 7, r = b >> 3;
    const int kt = r % A.nkt;
    const int tt = (r / A.nkt) * 8 + xcd;
    if (tt >= A.ntt) return;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int li = lane & 31, lh = lane >> 5;

    const int a_row = tid / A_C4, a_c4 = tid % A_C4;
    const int b_row = tid / B_C4, b_c4 = tid % B_C4;

    float4 ra[A_PASS], rb[B_PASS];

    auto load_global = [&](int p, int j) {
        const DevPlaneEntry e = PT.e[p];
        const float* Up = U + (size_t)e.u_off64 * 64 + (size_t)(kt * KT + a_row) * e.Lpad + j * LC + a_c4 * 4;
        const float* Vp = V + (size_t)e.v_off64 * 64 + (size_t)(j * LC + b_row) * A.Tpad + tt * TT + b_c4 * 4;
#pragma unroll
        for (int i = 0; i < A_PASS; ++i) ra[i] = *reinterpret_cast<const float4*>(Up + (size_t)i * A_ROWS * e.Lpad);
#pragma unroll
        for (int i = 0; i < B_PASS; ++i) rb[i] = *reinterpret_cast<const float4*>(Vp + (size_t)i * B_ROWS * A.Tpad);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PASS; ++i)
            *reinterpret_cast<float4*>(&As[buf][(a_row + i * A_ROWS) * AS + a_c4 * 4]) = ra[i];
#pragma unroll
        for (int i = 0; i < B_PASS; ++i)
            *reinterpret_cast<float4*>(&Bs[buf][(b_row + i * B_ROWS) * BS + b_c4 * 4]) = rb[i];
    };

    floatx16 acc[WM][WN];
    floatx16 Y[WM][WN][4];
#pragma unroll
    for (int mi = 0; mi < WM; ++mi)
#pragma unroll
        for (int nj = 0; nj < WN; ++nj) {
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mi][nj][e] = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 16; ++e) Y[mi][nj][q][e] = 0.f;
        }

    int p = 0, j = 0, buf = 0;
    int nch = PT.e[0].Lpad / LC;
    load_global(0, 0);
    store_lds(0);
    __syncthreads();

    while (true) {
        int pn = p, jn = j + 1;
        if (jn == nch) { pn = p + 1; jn = 0; }
        const bool has_next = pn < PT.n;
        if (has_next) load_global(pn, jn);

        const float* as = &As[buf][(wave_m * 32 * WM + li) * AS + 4 * lh];
        const float* bs = &Bs[buf][(4 * lh) * BS + wave_n * 32 * WN + li];
#pragma unroll
        for (int g = 0; g < LC / 8; ++g) {
            float4 av[WM];
#pragma unroll
            for (int mi = 0; mi < WM; ++mi) av[mi] = *reinterpret_cast<const float4*>(as + mi * 32 * AS + 8 * g);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                float bv[WN];
#pragma unroll
                for (int nj = 0; nj < WN; ++nj) bv[nj] = bs[(8 * g + s) * BS + nj * 32];
#pragma unroll
                for (int mi = 0; mi < WM; ++mi) {
                    const float a_s = s == 0 ? av[mi].x : s == 1 ? av[mi].y : s == 2 ? av[mi].z : av[mi].w;
#pragma unroll
                    for (int nj = 0; nj < WN; ++nj)
                        acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_s, bv[nj], acc[mi][nj], 0, 0, 0);
                }
            }
        }

        if (has_next) store_lds(buf ^ 1);
        __syncthreads();

        if (jn == 0) {
            // plane p complete: fold M_p into the 2x2 outputs with its +-1/0 pattern
            const int coef = PT.e[p].coef;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cq = (coef >> (2 * q)) & 3;
                if (cq != 0) {
                    const float sg = cq == 1 ? 1.f : -1.f;
#pragma unroll
                    for (int mi = 0; mi < WM; ++mi)
#pragma unroll
                        for (int nj = 0; nj < WN; ++nj)
#pragma unroll
                            for (int e = 0; e < 16; ++e)
                                Y[mi][nj][q][e] = fmaf(sg, acc[mi][nj][e], Y[mi][nj][q][e]);
                }
            }
#pragma unroll
            for (int mi = 0; mi < WM; ++mi)
#pragma unroll
                for (int nj = 0; nj < WN; ++nj)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[mi][nj][e] = 0.f;
            if (!has_next) break;
            nch = PT.e[pn].Lpad / LC;
        }
        p = pn; j = jn; buf ^= 1;
    }

    // Scatter: lane holds column t (li) and rows k = 8*(e/4) + 4*lh + e%4 of each 32x32 block.
    const int tiles = A.TH * A.TW;
    const bool pair_ok = (A.OW & 1) == 0;
#pragma unroll
    for (int nj = 0; nj < WN; ++nj) {
        const int t = tt * TT + wave_n * 32 * WN + nj * 32 + li;
        if (t >= A.T) continue;
        const int n = t / tiles, rem = t - n * tiles;
        const int ty = rem / A.TW, tx = rem - ty * A.TW;
        const int oh = 2 * ty, ow = 2 * tx;
#pragma unroll
        for (int mi = 0; mi < WM; ++mi) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int k = kt * KT + wave_m * 32 * WM + mi * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
                if (k >= A.K) continue;
                float* yp = y + (((size_t)n * A.K + k) * A.OH + oh) * A.OW + ow;
                const float y00 = Y[mi][nj][0][e], y01 = Y[mi][nj][1][e];
                const float y10 = Y[mi][nj][2][e], y11 = Y[mi][nj][3][e];
                if (pair_ok) {
                    *reinterpret_cast<float2*>(yp) = make_float2(y00, y01);
                    if (oh + 1 < A.OH) *reinterpret_cast<float2*>(yp + A.OW) = make_float2(y10, y11);
                } else {
                    yp[0] = y00;
                    if (ow + 1 < A.OW) yp[1] = y01;
                    if (oh + 1 < A.OH) {
                        yp[A.OW] = y10;
                        if (ow + 1 < A.OW) yp[A.OW + 1] = y11;
                    }
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

dwm_status_t launch_filter_transform(const dwm_plan& p, const float* w, float* U, void* stream)
{
    dim3 grid((p.d.rows_total + 255) / 256, p.d.Kpad), block(256);
    hipLaunchKernelGGL(filter_transform_kernel, grid, block, 0, (hipStream_t)stream, p.d, w, U);
    return check_launch();
}

dwm_status_t launch_input_transform(const dwm_plan& p, const float* x, float* V, void* stream)
{
    if (p.d.rows_total > 65535) return DWM_ERR_UNSUPPORTED;
    dim3 grid(p.d.Tpad / 256, p.d.rows_total), block(256);
    hipLaunchKernelGGL(input_transform_gather_kernel, grid, block, 0, (hipStream_t)stream, p.d, x, V);
    return check_launch();
}

template <int WM, int WN, int LC>
static dwm_status_t launch_contract(const dwm_plan& p, const float* U, const float* V, float* y, void* stream)
{
    constexpr int KT = 64 * WM, TT = 64 * WN;
    static_assert(kKAlign % KT == 0 && kTAlign % TT == 0 && kLAlign % LC == 0, "padding must cover the tile");
    ContractArgs a;
    a.K = p.d.K; a.T = p.d.T; a.Kpad = p.d.Kpad; a.Tpad = p.d.Tpad;
    a.OH = p.d.OH; a.OW = p.d.OW; a.TH = p.d.TH; a.TW = p.d.TW;
    a.nkt = (p.d.K + KT - 1) / KT;
    a.ntt = (p.d.T + TT - 1) / TT;
    const long long blocks = 8LL * a.nkt * ((a.ntt + 7) / 8);
    if (blocks > 0x7fffffffLL) return DWM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((contract_output_kernel<WM, WN, LC>), dim3((unsigned)blocks), dim3(256), 0,
                       (hipStream_t)stream, a, p.planes, U, V, y);
    return check_launch();
}

dwm_status_t launch_contract_output(const dwm_plan& p, const float* U, const float* V, float* y, void* stream)
{
    const int v = p.variant_contract < 0 ? 0 : p.variant_contract;
    switch (v) {
        case 0: return launch_contract<1, 1, 16>(p, U, V, y, stream);
        case 1: return launch_contract<2, 1, 16>(p, U, V, y, stream);
        case 2: return launch_contract<1, 2, 16>(p, U, V, y, stream);
        case 3: return launch_contract<2, 2, 16>(p, U, V, y, stream);
        default: return DWM_ERR_INVALID_ARG;
    }
}

}  // namespace dwm
