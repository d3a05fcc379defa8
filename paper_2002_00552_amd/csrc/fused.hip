// Single-kernel forward path of libdwm for layers with few input channels (gfx950).
//
// All five steps of the paper's Sec. 4.1 list run in one launch; nothing but x, U and y
// touches HBM.  It applies when the input footprint of a block of up to 64 output tiles,
// ALL channels, fits in LDS and every class's reduction length L = parts*C is at most 32
// (stem layers: C = 3).  For such layers the staged path is bound by the round trip of V
// through HBM (V is m/4 times larger than y's share of x), which this path removes -- the
// fusion the paper names as future work (Sec. 5.3, last paragraph).
//
// A workgroup owns a BH x BW block of 2x2 output tiles of one image (64 lanes of tiles)
// and 32*WGM filters; it has 2*WGM waves, each owning 32 filters x 32 tiles.
//   1. "Splitting" of the input: the block's padded input region is staged once in LDS,
//      zero padding written explicitly, columns de-interleaved modulo 2*stride (adjacent
//      tiles' patches of a polyphase view are then adjacent words).
//   2. "Transformation": for one class and one row frequency fh at a time, every wave
//      builds rows l = slot*C + c of V = B^T d B for the (lw+1) planes (fh, 0..lw) into LDS.
//   3. "Calculation": per plane, ceil(L/2) v_mfma_f32_32x32x2_f32.  The A operand comes
//      straight from L2 into registers, one plane ahead, out of the transposed copy
//      UT[plane][l][k] (32 consecutive filters per half wave: fully coalesced).
//   4. "Detransformation" + "Aggregation": the accumulator is folded into four running
//      2x2 outputs with the plane's 0/+-1 pattern; y is written once at the end.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "plan.hpp"

namespace dwm {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Row f of B^T of F(2,l) as sa*d[ia] + sb*d[ib] (sb = 0: single term).
__device__ __forceinline__ void bt_row(int l, int f, int& ia, float& sa, int& ib, float& sb)
{
    ia = 0; ib = 0; sa = 1.f; sb = 0.f;
    if (l == 3) {
        if (f == 0) { ia = 0; ib = 2; sb = -1.f; }
        else if (f == 1) { ia = 1; ib = 2; sb = 1.f; }
        else if (f == 2) { ia = 2; ib = 1; sb = -1.f; }
        else { ia = 1; ib = 3; sb = -1.f; }
    } else if (l == 2) {
        if (f == 0) { ia = 0; ib = 1; sb = -1.f; }
        else if (f == 1) { ia = 1; }
        else { ia = 2; ib = 1; sb = -1.f; }
    } else {
        ia = f;
    }
}

template <int LW>
__device__ __forceinline__ void bt_cols(const float v[4], float o[4])
{
    if (LW == 3) {
        o[0] = v[0] - v[2]; o[1] = v[1] + v[2]; o[2] = v[2] - v[1]; o[3] = v[1] - v[3];
    } else if (LW == 2) {
        o[0] = v[0] - v[1]; o[1] = v[1]; o[2] = v[2] - v[1];
    } else {
        o[0] = v[0]; o[1] = v[1];
    }
}

// One V row (all lanes = all tiles of the block) for the planes (fh, 0..LW); ra/rb are the
// LDS offsets of the two patch rows that B^T row fh combines, co those of the patch columns.
template <int LW>
__device__ __forceinline__ void build_row(const float* __restrict__ xt, int ra, float sa, int rb, float sb,
                                          const int4 co, float* __restrict__ vrow, int plane_floats)
{
    const int cof[4] = {co.x, co.y, co.z, co.w};
    float v[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
#pragma unroll
    for (int b = 0; b <= LW; ++b) v[b] = sa * xt[ra + cof[b]] + sb * xt[rb + cof[b]];
    bt_cols<LW>(v, o);
#pragma unroll
    for (int b = 0; b <= LW; ++b) vrow[b * plane_floats] = o[b];
}

// MFMA chain of one plane with a compile-time length (no compares or branches inside).
template <int NM, int NA>
__device__ __forceinline__ void mfma_chain(const float (&a)[NA], const float (&bv)[NA], floatx16& acc)
{
    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], bv[0], zero, 0, 0, 0);
#pragma unroll
    for (int m = 1; m < NM; ++m)
        if (m < NA) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[m], bv[m], acc, 0, 0, 0);
}

// WGM: K blocks of 32 per workgroup.  NA: operand slots per plane, >= ceil(L/2) of every class;
// every plane loads NA operands (rows past its own belong to the next plane and are ignored),
// so the number of loads in flight is a compile-time constant.
template <int WGM, int NA>
__global__ __launch_bounds__(128 * WGM, WGM == 1 ? 4 : WGM == 2 ? 3 : 1) void fused_forward_kernel(
    DevPlan P, FusedArgs F, PlaneTable PT, const float* __restrict__ x, const float* __restrict__ U,
    float* __restrict__ y)
{
    constexpr int NW = 2 * WGM, NT = 64 * NW;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    // LDS: per-plane info | per-row info | staged input | two V buffers
    int4* pinfo = reinterpret_cast<int4*>(lds);                 // [kMaxPlanes + 1]
    int4* rowinfo = pinfo + (kMaxPlanes + 1);                   // [rows_all][2]: patch row / column offsets
    float* xs = reinterpret_cast<float*>(rowinfo + 2 * F.rows_all);  // [C][nrows][nphase][lwp]
    float* Vs = xs + P.C * F.chan_floats;                       // 2 x [4 planes][vrows][64]
    const int plane_floats = F.vrows * 64;
    const int vbuf_floats = 4 * plane_floats;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int li = lane & 31, lh = lane >> 5;

    const int b = blockIdx.x;
    const int btx = b % F.nbw, bty = (b / F.nbw) % F.nbh, n = b / (F.nbw * F.nbh);
    const int ty0 = bty * F.BH, tx0 = btx * F.BW;
    const int k0 = (blockIdx.y * WGM + wave_m) * 32;

    // ---- 0. tables: everything the loops below need per plane and per V row, looked up once ----
    for (int p = tid; p <= PT.n; p += NT) {
        int4 v = make_int4(0, 0, 0, -1);
        if (p < PT.n) {
            int qi = 0;
            while (qi + 1 < P.ncls && p >= P.cls[qi + 1].plane0) ++qi;
            const DevClass q = P.cls[qi];
            const int r = p - q.plane0, fh = r / (q.lw + 1), fw = r - fh * (q.lw + 1);
            // the group after this plane's group (built while this group is multiplied)
            int gqi = qi, gfh = fh + 1;
            if (gfh > q.lh) { gfh = 0; ++gqi; }
            const int next_group = (fw == 0 && gqi < P.ncls) ? (gqi << 8 | gfh) : -1;
            v.x = (q.Lt >> 1) | fw << 8 | (fw == q.lw ? 1 << 16 : 0);  // MFMAs, plane in group, last of group
            v.y = PT.e[p].coef;
            v.z = (int)PT.e[p].ut_off64;
            v.w = next_group;
        } else {
            v.x = 1;
        }
        pinfo[p] = v;
    }
    for (int r = tid; r < F.rows_all; r += NT) {
        int qi = 0;
        while (qi + 1 < P.ncls && r >= F.row0[qi + 1]) ++qi;
        const DevClass q = P.cls[qi];
        const int l = r - F.row0[qi];
        int4 ro = make_int4(0, 0, 0, 0), co = make_int4(0, 0, 0, 0);
        if (l < q.L) {
            const int slot = l / P.C, c = l - slot * P.C;
            const int ah = slot / q.wn, bw = slot - ah * q.wn;
            const int* rr = F.roff[q.h0 + ah];
            const int* cc = F.coff[q.w0 + bw];
            const int base = c * F.chan_floats;
            ro = make_int4(base + rr[0], base + rr[1], base + rr[2], base + rr[3]);
            co = make_int4(cc[0], cc[1], cc[2], cc[3]);
        }
        rowinfo[2 * r] = ro;
        rowinfo[2 * r + 1] = co;
    }

    // ---- 1. stage the block's input region (padded coordinates), a wave per row ----
    {
        const int prow0 = 2 * ty0 * P.s - P.P, pcol0 = 2 * tx0 * P.s - P.P;
        const float* xn = x + (size_t)n * P.C * P.H * P.W;
        for (int cr = wave; cr < P.C * F.nrows; cr += NW) {
            const int c = cr / F.nrows, r = cr - c * F.nrows;
            const int ih = prow0 + r;
            const bool row_ok = ih >= 0 && ih < P.H;
            const float* xr = xn + ((size_t)c * P.H + ih) * P.W + pcol0;
            float* xsr = xs + c * F.chan_floats + r * F.row_floats;
            for (int col = lane; col < F.lw_in; col += 64) {
                const int iw = pcol0 + col;
                const float v = (row_ok && iw >= 0 && iw < P.W) ? xr[col] : 0.f;
                const int idx = F.div_nphase.div(col);
                xsr[(col - idx * F.nphase) * F.lwp + idx] = v;
            }
        }
    }

    // this lane's tile in the build phase (lane = tile of the block; idle lanes reuse tile 0)
    const float* xt;
    {
        const int by = F.div_bw.div(lane), bx = lane - by * F.BW;
        xt = xs + (by < F.BH ? by * F.tile_row_step + bx : 0);
    }

    floatx16 acc, Y[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) Y[q][e] = 0.f;

    // ---- 2. V rows of the planes (fh, 0..lw) of class qi into buffer vb ----
    auto build_group = [&](int qi, int fh, float* vb) {
        const int lhq = P.cls[qi].lh, lwq = P.cls[qi].lw, Lq = P.cls[qi].L, Ltq = P.cls[qi].Lt;
        const int4* ri = rowinfo + 2 * F.row0[qi];
        int ia, ib;
        float sa, sb;
        bt_row(lhq, fh, ia, sa, ib, sb);
        auto one_row = [&](int l) {
            float* vrow = vb + l * 64 + (lane ^ ((l & 1) << 5));
            if (l < Lq) {
                const int* rr = reinterpret_cast<const int*>(ri + 2 * l);
                const int ra = rr[ia], rb = rr[ib];
                const int4 co = ri[2 * l + 1];
                if (lwq == 3) build_row<3>(xt, ra, sa, rb, sb, co, vrow, plane_floats);
                else if (lwq == 2) build_row<2>(xt, ra, sa, rb, sb, co, vrow, plane_floats);
                else build_row<1>(xt, ra, sa, rb, sb, co, vrow, plane_floats);
            } else {
                for (int bq = 0; bq <= lwq; ++bq) vrow[bq * plane_floats] = 0.f;
            }
        };
        int l = wave;
        for (; l + NW < Ltq; l += 2 * NW) {  // two rows in flight per wave
            one_row(l);
            one_row(l + NW);
        }
        if (l < Ltq) one_row(l);
    };

    // A operand of plane p: lane (i, h) needs UT_p[2m+h][k0+i] for MFMA m -- 32 consecutive
    // filters per half wave, read straight from L2 into registers one plane ahead.
    const size_t a_step = (size_t)2 * P.Kpad;
    auto load_a = [&](unsigned ut_off64, float (&a)[NA]) {
        const float* ut = U + (size_t)ut_off64 * 64 + (size_t)lh * P.Kpad + k0 + li;
#pragma unroll
        for (int m = 0; m < NA; ++m) a[m] = ut[m * a_step];
    };

    // ---- 3./4. one plane: MFMA over its reduction, fold into the 2x2 outputs ----
    auto do_plane = [&](int coef, int nm, const float* vplane, const float (&a)[NA]) {
        const float* bs = vplane + lh * 64 + ((wave_n * 32 + li) ^ (lh << 5));
        float bv[NA];
#pragma unroll
        for (int m = 0; m < NA; ++m) bv[m] = bs[m * 128];
        switch (nm) {
            case 1: mfma_chain<1, NA>(a, bv, acc); break;
            case 2: mfma_chain<2, NA>(a, bv, acc); break;
            case 3: mfma_chain<3, NA>(a, bv, acc); break;
            case 4: mfma_chain<4, NA>(a, bv, acc); break;
            case 5: mfma_chain<5, NA>(a, bv, acc); break;
            case 6: mfma_chain<6, NA>(a, bv, acc); break;
            case 7: mfma_chain<7, NA>(a, bv, acc); break;
            case 8: mfma_chain<8, NA>(a, bv, acc); break;
            case 9: mfma_chain<9, NA>(a, bv, acc); break;
            case 10: mfma_chain<10, NA>(a, bv, acc); break;
            case 11: mfma_chain<11, NA>(a, bv, acc); break;
            case 12: mfma_chain<12, NA>(a, bv, acc); break;
            case 13: mfma_chain<13, NA>(a, bv, acc); break;
            case 14: mfma_chain<14, NA>(a, bv, acc); break;
            case 15: mfma_chain<15, NA>(a, bv, acc); break;
            default: mfma_chain<16, NA>(a, bv, acc); break;
        }
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
            const int cq = (coef >> (2 * qq)) & 3;
            if (cq != 0) {
                const float sg = cq == 1 ? 1.f : -1.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) Y[qq][e] = fmaf(sg, acc[e], Y[qq][e]);
            }
        }
    };

    // Groups (class, fh) are walked in plane order; V of group g+1 is built before the MFMAs
    // of group g (two V buffers), so one barrier per group suffices and the waves of a SIMD
    // overlap building with multiplying.
    float a0[NA], a1[NA];
    __syncthreads();  // tables and staged input complete
    build_group(0, 0, Vs);
    int4 cur = pinfo[0];
    load_a((unsigned)cur.z, a0);
    __syncthreads();
    int vsel = 0;
    auto step = [&](int p, const float (&a_use)[NA], float (&a_load)[NA]) {
        const int4 nxt = pinfo[p + 1];  // the entry after the last plane is a harmless dummy
        if (cur.w >= 0) build_group(cur.w >> 8, cur.w & 255, Vs + (vsel ^ 1) * vbuf_floats);
        load_a((unsigned)(p + 1 < PT.n ? nxt.z : cur.z), a_load);
        do_plane(cur.y, cur.x & 255, Vs + vsel * vbuf_floats + ((cur.x >> 8) & 255) * plane_floats, a_use);
        if (cur.x >> 16) {  // last plane of the group
            __syncthreads();
            vsel ^= 1;
        }
        cur = nxt;
    };
    for (int p = 0; p < PT.n; p += 2) {
        step(p, a0, a1);
        if (p + 1 < PT.n) step(p + 1, a1, a0);
    }

    // ---- scatter: lane holds tile t = wave_n*32 + li and filters k0 + 8*(e/4) + 4*lh + e%4 ----
    const int t = wave_n * 32 + li;
    const int by = F.div_bw.div(t), bx = t - by * F.BW;
    const int ty = ty0 + by, tx = tx0 + bx;
    if (by >= F.BH || ty >= P.TH || tx >= P.TW) return;
    const int oh = 2 * ty, ow = 2 * tx;
    const bool pair_ok = (P.OW & 1) == 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int k = k0 + 8 * (e >> 2) + 4 * lh + (e & 3);
        if (k >= P.K) continue;
        float* yp = y + (((size_t)n * P.K + k) * P.OH + oh) * P.OW + ow;
        if (pair_ok) {
            *reinterpret_cast<float2*>(yp) = make_float2(Y[0][e], Y[1][e]);
            if (oh + 1 < P.OH) *reinterpret_cast<float2*>(yp + P.OW) = make_float2(Y[2][e], Y[3][e]);
        } else {
            yp[0] = Y[0][e];
            if (ow + 1 < P.OW) yp[1] = Y[1][e];
            if (oh + 1 < P.OH) {
                yp[P.OW] = Y[2][e];
                if (ow + 1 < P.OW) yp[P.OW + 1] = Y[3][e];
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Host: does the path apply, and with which block of tiles
// ---------------------------------------------------------------------------------
bool fused_setup(const dwm_plan& p, FusedArgs* out)
{
    const DevPlan& d = p.d;
    FusedArgs f{};
    int max_L = 0;
    for (int i = 0; i < d.ncls; ++i) max_L = std::max(max_L, d.cls[i].L);
    if (max_L > 32) return false;
    int max_oh = 0, max_ow = 0;
    for (int i = 0; i < d.nh; ++i) max_oh = std::max(max_oh, d.s * (d.ph[i].j + d.ph[i].l) + d.ph[i].p);
    for (int i = 0; i < d.nw; ++i) max_ow = std::max(max_ow, d.s * (d.pw[i].j + d.pw[i].l) + d.pw[i].p);
    f.nphase = 2 * d.s;
    f.vrows = (max_L + 1) & ~1;
    const int wgm = d.K <= 32 ? 1 : d.K <= 64 ? 2 : d.K <= 96 ? 3 : 4;
    // two V buffers of [4][vrows][64], plus 2*NA rows of slack: every plane reads a fixed number
    // of operand rows, the surplus ones run into the next plane (or the slack) and are ignored
    const int na = f.vrows <= 8 ? 4 : f.vrows <= 16 ? 8 : 16;
    const size_t v_bytes = (size_t)(2 * 4 * f.vrows + 2 * na) * 64 * sizeof(float);
    const size_t budget = 128 * 1024;  // staged input + V and U buffers per workgroup

    // block of tiles: most useful lanes first, then the smallest staged region
    double best_eff = 0.0;
    size_t best_x = 0;
    for (int bw = 1; bw <= 64 && bw <= d.TW; ++bw) {
        int bh = 64 / bw;
        if (bh > d.TH) bh = d.TH;
        if (bh < 1) continue;
        const int nbh = (d.TH + bh - 1) / bh, nbw = (d.TW + bw - 1) / bw;
        const double eff = (double)d.TH * d.TW / ((double)nbh * nbw * 64);
        const int nrows = 2 * d.s * (bh - 1) + max_oh + 1;
        const int lw_in = 2 * d.s * (bw - 1) + max_ow + 1;
        const int lwp = ((lw_in + f.nphase - 1) / f.nphase) | 1;
        const size_t x_bytes = (size_t)d.C * nrows * f.nphase * lwp * sizeof(float);
        if (x_bytes + v_bytes > budget) continue;
        if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && x_bytes < best_x)) {
            best_eff = eff; best_x = x_bytes;
            f.BH = bh; f.BW = bw; f.nbh = nbh; f.nbw = nbw;
            f.nrows = nrows; f.lw_in = lw_in; f.lwp = lwp;
        }
    }
    if (best_eff < 0.5) return false;
    if ((long long)d.N * f.nbh * f.nbw > 0x7fffffffLL) return false;
    f.row_floats = f.nphase * f.lwp;
    f.chan_floats = f.nrows * f.row_floats;
    f.tile_row_step = 2 * d.s * f.row_floats;
    f.wgm = wgm;
    f.nkt = (d.K + 32 * f.wgm - 1) / (32 * f.wgm);
    if (f.nkt > 65535) return false;
    f.div_bw.init((unsigned)f.BW);
    f.div_nphase.init((unsigned)f.nphase);
    f.div_c.init((unsigned)d.C);
    for (int i = 0; i < kMaxPieces; ++i)
        for (int k = 0; k < 4; ++k) {
            const int oh = i < d.nh ? d.s * (d.ph[i].j + k) + d.ph[i].p : 0;
            const int ow = i < d.nw ? d.s * (d.pw[i].j + k) + d.pw[i].p : 0;
            f.roff[i][k] = oh * f.row_floats;
            f.coff[i][k] = (ow % f.nphase) * f.lwp + ow / f.nphase;
        }
    f.rows_all = 0;
    for (int i = 0; i < d.ncls; ++i) {
        f.row0[i] = f.rows_all;
        f.rows_all += (d.cls[i].L + 1) & ~1;
    }
    f.lds_bytes = (size_t)(kMaxPlanes + 1 + 2 * f.rows_all) * 16 + best_x + v_bytes;
    *out = f;
    return true;
}

template <int WGM, int NA>
static dwm_status_t launch_fused(const dwm_plan& p, const float* x, const float* U, float* y, void* stream)
{
    const FusedArgs& f = p.fused;
    auto kernel = fused_forward_kernel<WGM, NA>;
    if (f.lds_bytes > 64 * 1024) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return DWM_ERR_HIP;
    }
    dim3 grid((unsigned)(p.d.N * f.nbh * f.nbw), (unsigned)f.nkt), block(128 * WGM);
    hipLaunchKernelGGL(kernel, grid, block, f.lds_bytes, (hipStream_t)stream, p.d, f, p.planes, x, U, y);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

template <int WGM>
static dwm_status_t launch_fused_na(const dwm_plan& p, const float* x, const float* U, float* y, void* stream)
{
    if (p.fused.vrows <= 8) return launch_fused<WGM, 4>(p, x, U, y, stream);
    if (p.fused.vrows <= 16) return launch_fused<WGM, 8>(p, x, U, y, stream);
    return launch_fused<WGM, 16>(p, x, U, y, stream);
}

dwm_status_t launch_fused_forward(const dwm_plan& p, const float* x, const float* U, float* y, void* stream)
{
    if (!p.fused_ok) return DWM_ERR_INVALID_ARG;
    switch (p.fused.wgm) {
        case 1: return launch_fused_na<1>(p, x, U, y, stream);
        case 2: return launch_fused_na<2>(p, x, U, y, stream);
        case 3: return launch_fused_na<3>(p, x, U, y, stream);
        default: return launch_fused_na<4>(p, x, U, y, stream);
    }
}

}  // namespace dwm
