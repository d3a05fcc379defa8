// Single-kernel forward path of libdwm (gfx950), for layers with few input channels.
//
// All five steps of the paper's Sec. 4.1 list run in one launch; only x, the transformed
// filter and y touch HBM, and the transformed input V never leaves the registers.
//
// A workgroup (four waves) owns a BH x BW block of 2x2 output tiles of one image; a wave
// owns 16 of those tiles and walks the filters 32 at a time ("slices").
//   1. "Splitting" of the input: the block's padded input region is staged once in LDS,
//      zero padding written explicitly, columns de-interleaved modulo 2*stride.
//   2. "Transformation" + "Calculation": the contraction runs on v_mfma_f32_16x16x4_f32,
//      whose B operand wants, from lane (n, q), the value V[row 4m+q][tile n] of the plane
//      being multiplied.  The lane reads the patch of ITS row (part, channel) and ITS tile
//      from LDS, applies B^T d B in registers, and holds all frequencies of that patch: they
//      are exactly its B operands for the planes (fh, fw) of step m.  The A operand -- the
//      transformed filter of 32 filters x 4 rows -- is one contiguous 512-byte read per plane
//      and step from a copy laid out for this kernel (L2 hits; every workgroup reads the same).
//      Every plane has its own accumulator (16 planes x 2 filter halves x 4 registers), so
//      nothing is folded until the reduction is over.
//   3. "Detransformation" + "Aggregation": A^T M A once per class and slice, in two stages,
//      straight from the accumulators into the 2x2 outputs, which are written once.
// Pieces of two and three taps share the four frequencies of F(2,3): a 2-tap piece is run
// as a 3-tap piece whose third tap is zero, so its fourth frequency vanishes on the filter
// side and is skipped (three multiplications, as the count of Table 3 assumes), and the
// input side needs only the first three patch values.  One-tap pieces (phases that hold a
// single tap) keep their two "frequencies" (no transform) in classes of their own.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "plan.hpp"

namespace dwm {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// (G_l g)[i] with the 2-tap case run as 3 taps with a zero third tap.
__device__ __forceinline__ float fused_g_row(int l, int i, float v0, float v1, float v2)
{
    if (l == 1) return v0;
    switch (i) {
        case 0: return v0;
        case 1: return 0.5f * (v0 + v1 + v2);
        case 2: return 0.5f * (v0 - v1 + v2);
        default: return v2;
    }
}

// ---------------------------------------------------------------------------------
// Filter copy for this path: UF[class][slice][plane][row][i][half], filter = 32*slice +
// 16*half + i; zero for filters >= K, padding rows and frequencies a part does not have.
// One thread per (row, filter).
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fused_filter_kernel(DevPlan P, FusedArgs F, const float* __restrict__ w,
                                                        float* __restrict__ U, int gap0, int gap1)
{
    // the alignment gap before this copy belongs to the filter buffer: it is written too
    if (blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = gap0 + threadIdx.x; i < gap1; i += blockDim.x) U[i] = 0.f;
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (row >= F.rows_total) return;
    int fi = 0;
    while (fi + 1 < F.nfc && row >= F.fc[fi + 1].row0) ++fi;
    const FusedClass fc = F.fc[fi];
    const unsigned desc = F.rowdesc[row];
    const bool real = (desc >> 15) != 0 && k < P.K;
    const DevPiece hp = P.ph[desc & 15], wp = P.pw[(desc >> 4) & 15];
    const int c = (desc >> 8) & 127;
    float g[3][3];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            float v = 0.f;
            if (real && i < hp.l && j < wp.l) {
                const int r = P.s * (hp.j + i) + hp.p, q = P.s * (wp.j + j) + wp.p;
                v = w[(((size_t)k * P.C + c) * P.R + r) * P.S + q];
            }
            g[i][j] = v;
        }
    float t[4][3];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j) t[i][j] = fused_g_row(hp.l, i, g[0][j], g[1][j], g[2][j]);
    const int slice = k >> 5, half = (k >> 4) & 1, ki = k & 15;
    float* dst = U + fc.uf_off + ((size_t)slice * fc.nfh * fc.nfw * fc.rows + (row - fc.row0)) * 32 + ki * 2 + half;
#pragma unroll
    for (int fh = 0; fh < 4; ++fh)
#pragma unroll
        for (int fw = 0; fw < 4; ++fw)
            if (fh < fc.nfh && fw < fc.nfw) {
                const float u = fused_g_row(wp.l, fw, t[fh][0], t[fh][1], t[fh][2]);
                dst[(size_t)(fh * fc.nfw + fw) * fc.rows * 32] = (real && fh <= hp.l && fw <= wp.l) ? u : 0.f;
            }
}

// ---------------------------------------------------------------------------------
// One class (a pair of families) for one slice of 32 filters: every step of four rows is
// patch from LDS -> B^T d B -> one MFMA per plane and filter half; then the output transform.
// WH, WW: 1 for the family of 2- and 3-tap pieces (F(2,3) frequencies), 0 for one-tap pieces.
// A step whose pieces have two taps skips the planes of the fourth frequency.
// ---------------------------------------------------------------------------------
template <int WIDE>
__device__ __forceinline__ void fused_bt(const float d[4], float o[4])
{
    if (WIDE) {  // B^T of F(2,3) (Sec. 3.2); with two taps o[3] is not used
        o[0] = d[0] - d[2];
        o[1] = d[1] + d[2];
        o[2] = d[2] - d[1];
        o[3] = d[1] - d[3];
    } else {
        o[0] = d[0];
        o[1] = d[1];
    }
}

// A operand of one plane and step: 512 contiguous bytes per wave, lane l takes bytes 8l..8l+7
// (filters i and 16+i of the slice, row 4*step + q; l = 16q + i).  A buffer load: the base is a
// scalar resource, the plane/step offset a scalar, the lane's offset a fixed register -- no
// vector instruction is spent on addresses.
typedef float fused_float2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float2 fused_load_a(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff)
{
    const fused_float2 v = __builtin_bit_cast(fused_float2, __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, soff, 0));
    return make_float2(v.x, v.y);
}

__device__ __forceinline__ void fused_mfma(float2 a, float bv, floatx4 (&acc)[2])
{
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, bv, acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, bv, acc[1], 0, 0, 0);
}

// A^T of the family: four frequencies (F(2,3), Sec. 3.2) or two (identity).
template <int WIDE>
__device__ __forceinline__ void fused_at(const floatx4 m[4], floatx4 o[2])
{
    if (WIDE) {
        o[0] = m[0] + m[1] + m[2];
        o[1] = m[1] - m[2] - m[3];
    } else {
        o[0] = m[0];
        o[1] = m[1];
    }
}

// Y[a][b][half] += sum AT_h[a][fh] AT_w[b][fw] acc[fh][fw][half]
template <int WH, int WW>
__device__ __forceinline__ void fused_output(const floatx4 (&acc)[WH ? 4 : 2][WW ? 4 : 2][2], floatx4 (&Y)[2][2][2])
{
    constexpr int NH = WH ? 4 : 2, NW = WW ? 4 : 2;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        floatx4 t[NH][2];  // [fh][b]
#pragma unroll
        for (int fh = 0; fh < NH; ++fh) {
            floatx4 m[4], o[2];
#pragma unroll
            for (int fw = 0; fw < 4; ++fw) m[fw] = acc[fh][fw < NW ? fw : 0][half];
            fused_at<WW>(m, o);
            t[fh][0] = o[0];
            t[fh][1] = o[1];
        }
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            floatx4 m[4], o[2];
#pragma unroll
            for (int fh = 0; fh < 4; ++fh) m[fh] = t[fh < NH ? fh : 0][b];
            fused_at<WH>(m, o);
            Y[0][b][half] += o[0];
            Y[1][b][half] += o[1];
        }
    }
}

// The lane's patch of one row: d[i][j] = staged input at (tile base) + (row's offset i, j).
template <int NH, int NW>
__device__ __forceinline__ void fused_read_patch(const float* __restrict__ xt, const int4* __restrict__ ri,
                                              float (&d)[NH][NW])
{
    const char* xb = reinterpret_cast<const char*>(xt);
#pragma unroll
    for (int i = 0; i < NH; ++i) {
        const int4 o = ri[i];
        d[i][0] = *reinterpret_cast<const float*>(xb + o.x);
        d[i][1] = *reinterpret_cast<const float*>(xb + o.y);
        if (NW == 4) {
            d[i][2] = *reinterpret_cast<const float*>(xb + o.z);
            d[i][3] = *reinterpret_cast<const float*>(xb + o.w);
        }
    }
}

// uf: the class's filter copy for this slice (the same for the whole wave); voff = 8 * lane.
template <int WH, int WW>
__device__ __forceinline__ void fused_class(const FusedArgs& F, const FusedClass& fc, const float* __restrict__ xt,
                                         const int4* __restrict__ ri, const float* __restrict__ uf, unsigned voff,
                                         floatx4 (&Y)[2][2][2])
{
    constexpr int NH = WH ? 4 : 2, NW = WW ? 4 : 2;
    floatx4 acc[NH][NW][2];
#pragma unroll
    for (int i = 0; i < NH; ++i)
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            acc[i][j][0] = floatx4{0.f, 0.f, 0.f, 0.f};
            acc[i][j][1] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    const unsigned plane_bytes = (unsigned)fc.rows * 32u * (unsigned)sizeof(float);
    // raw buffer over the class's copy for this slice (at most nfh*nfw*rows*128 bytes)
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(uf), 0, (int)(plane_bytes * (unsigned)(NH * NW)), 0x00020000);
    // A operands travel one step ahead: a plane's registers are refilled for the next step as
    // soon as its MFMAs of this step are issued (the last step refills with itself).
    float2 a[NH][NW];
#pragma unroll
    for (int i = 0; i < NH; ++i)
#pragma unroll
        for (int j = 0; j < NW; ++j) a[i][j] = fused_load_a(rsrc, voff, (unsigned)(i * NW + j) * plane_bytes);
    int type = F.step_type[fc.step0];
    // the patch of the NEXT step is read from LDS before this step's MFMAs are issued; a row's
    // 16 patch offsets (bytes, channel included) come from the table, the lane's tile base is added
    // (two patch buffers that swap roles from step to step: the loop body is written twice)
    float d0[NH][NW], d1[NH][NW];
    fused_read_patch<NH, NW>(xt, ri, d0);
    auto step = [&](int st, const float (&d)[NH][NW], float (&dn)[NH][NW]) {
        const bool h3 = !WH || (type >> 2) == 3, w3 = !WW || (type & 3) == 3;  // fourth frequency present
        const int nst = st + 1 < fc.nsteps ? st + 1 : st;
        type = F.step_type[fc.step0 + nst];
        const unsigned un = (unsigned)nst * 512u;
        fused_read_patch<NH, NW>(xt, ri + 16 * nst, dn);
        float tmp[NH][NW];
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            float col[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
#pragma unroll
            for (int i = 0; i < NH; ++i) col[i] = d[i][j];
            fused_bt<WH>(col, o);
#pragma unroll
            for (int i = 0; i < NH; ++i) tmp[i][j] = o[i];
        }
        float v[NH][NW];
#pragma unroll
        for (int i = 0; i < NH; ++i) {
            float rowv[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
#pragma unroll
            for (int j = 0; j < NW; ++j) rowv[j] = tmp[i][j];
            fused_bt<WW>(rowv, o);
#pragma unroll
            for (int j = 0; j < NW; ++j) v[i][j] = o[j];
        }
        constexpr int CH = WH ? 3 : 2, CW = WW ? 3 : 2;  // frequencies every piece of the family has
#pragma unroll
        for (int i = 0; i < CH; ++i)
#pragma unroll
            for (int j = 0; j < CW; ++j) {
                fused_mfma(a[i][j], v[i][j], acc[i][j]);
                a[i][j] = fused_load_a(rsrc, voff, un + (unsigned)(i * NW + j) * plane_bytes);
            }
        if (WW) {
            if (w3) {
#pragma unroll
                for (int i = 0; i < CH; ++i) fused_mfma(a[i][NW - 1], v[i][NW - 1], acc[i][NW - 1]);
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) a[i][NW - 1] = fused_load_a(rsrc, voff, un + (unsigned)(i * NW + 3) * plane_bytes);
        }
        if (WH) {
            if (h3) {
#pragma unroll
                for (int j = 0; j < CW; ++j) fused_mfma(a[NH - 1][j], v[NH - 1][j], acc[NH - 1][j]);
                if (WW && w3) fused_mfma(a[NH - 1][NW - 1], v[NH - 1][NW - 1], acc[NH - 1][NW - 1]);
            }
#pragma unroll
            for (int j = 0; j < NW; ++j) a[NH - 1][j] = fused_load_a(rsrc, voff, un + (unsigned)(3 * NW + j) * plane_bytes);
        }
    };
    int st = 0;
    for (; st + 1 < fc.nsteps; st += 2) {
        step(st, d0, d1);
        step(st + 1, d1, d0);
    }
    if (st < fc.nsteps) step(st, d0, d1);
    fused_output<WH, WW>(acc, Y);
}

// MULTI: the layer has more than one class, so their outputs are summed in Y; with a single
// class (no one-tap pieces) the registers of Y are saved: the class's output is the result.
template <bool MULTI>
__global__ __launch_bounds__(256, 2) void fused_forward_kernel(DevPlan P, FusedArgs F, const float* __restrict__ x,
                                                            const float* __restrict__ U, float* __restrict__ y)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    // LDS: per-row patch offsets | staged input
    int4* rowinfo = reinterpret_cast<int4*>(lds);                      // [rows_total][4]: byte offsets [i][j]
    float* xs = reinterpret_cast<float*>(rowinfo + 4 * F.rows_total);  // [C][nrows][nphase][lwp]

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 15, lq = lane >> 4;

    const int b = blockIdx.x;
    const int btx = b % F.nbw, bty = (b / F.nbw) % F.nbh, n = b / (F.nbw * F.nbh);
    const int ty0 = bty * F.BH, tx0 = btx * F.BW;

    // ---- 0. per-row patch offsets (row = part x channel), looked up once ----
    for (int r = tid; r < F.rows_total; r += 256) {
        const unsigned desc = F.rowdesc[r];
        const int base = (int)((desc >> 8) & 127) * F.chan_floats;
        const int* rr = F.roff[desc & 15];
        const int* cc = F.coff[(desc >> 4) & 15];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            rowinfo[4 * r + i] = make_int4(4 * (base + rr[i] + cc[0]), 4 * (base + rr[i] + cc[1]),
                                           4 * (base + rr[i] + cc[2]), 4 * (base + rr[i] + cc[3]));
    }

    // ---- 1. stage the block's input region (padded coordinates).  A unit is (channel, 8 rows);
    // a wave issues the loads of up to four units before it writes any of them to LDS. ----
    {
        const int prow0 = 2 * ty0 * P.s - P.Ph, pcol0 = 2 * tx0 * P.s - P.Pw;
        const float* xn = x + (size_t)n * P.C * P.H * P.W;
        const int nb8 = (F.nrows + 7) >> 3, units = P.C * nb8;
        for (int cb = 0; cb < F.lw_in; cb += 64) {
            const int col = cb + lane, iw = pcol0 + col;
            const bool iw_ok = iw >= 0 && iw < P.W;
            const int iwc = min(max(iw, 0), P.W - 1);
            const int idx = F.div_nphase.div(col);
            const int dcol = (col - idx * F.nphase) * F.lwp + idx;
            if (col < F.lw_in) {
                for (int u0 = wave; u0 < units; u0 += 16) {
                    float v[4][8];
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int u = min(u0 + 4 * g, units - 1);
                        const int c = u / nb8, r0 = (u - c * nb8) * 8;
                        const float* xc = xn + (size_t)c * P.H * P.W + iwc;
#pragma unroll
                        for (int k = 0; k < 8; ++k)
                            v[g][k] = xc[(size_t)min(max(prow0 + r0 + k, 0), P.H - 1) * P.W];
                    }
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int u = u0 + 4 * g;
                        if (u < units) {
                            const int c = u / nb8, r0 = (u - c * nb8) * 8;
                            float* xd = xs + c * F.chan_floats + dcol;
#pragma unroll
                            for (int k = 0; k < 8; ++k) {
                                const int ih = prow0 + r0 + k;
                                if (r0 + k < F.nrows)
                                    xd[(r0 + k) * F.row_floats] = (iw_ok && ih >= 0 && ih < P.H) ? v[g][k] : 0.f;
                            }
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

    // this lane's tile: number wave*16 + ln of the block (idle lanes reuse tile 0 and store nothing)
    const int tl = wave * 16 + ln;
    const int by = F.div_bw.div(tl), bx = tl - by * F.BW;
    const int ty = ty0 + by, tx = tx0 + bx;
    const bool tile_ok = by < F.BH && ty < P.TH && tx < P.TW;
    const float* xt = xs + (by < F.BH ? by * F.tile_row_step + bx : 0);

    const int slice0 = blockIdx.y * F.slices_per_wg;
    const int slice1 = min(slice0 + F.slices_per_wg, F.nslices);
    for (int ks = slice0; ks < slice1; ++ks) {
        floatx4 Y[2][2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int h = 0; h < 2; ++h) Y[a][c][h] = floatx4{0.f, 0.f, 0.f, 0.f};

        for (int fi = 0; fi < (MULTI ? F.nfc : 1); ++fi) {
            const FusedClass fc = F.fc[fi];
            const float* uf = U + fc.uf_off + (size_t)ks * fc.nfh * fc.nfw * fc.rows * 32;
            const int4* ri = rowinfo + 4 * (fc.row0 + lq);
            const unsigned voff = (unsigned)lane * 8u;
            if (fc.wide_h) {
                if (fc.wide_w) fused_class<1, 1>(F, fc, xt, ri, uf, voff, Y);
                else fused_class<1, 0>(F, fc, xt, ri, uf, voff, Y);
            } else {
                if (fc.wide_w) fused_class<0, 1>(F, fc, xt, ri, uf, voff, Y);
                else fused_class<0, 0>(F, fc, xt, ri, uf, voff, Y);
            }
        }

        // ---- scatter: lane (ln, lq) holds tile ln and filters 32*ks + 16*half + 4*lq + r ----
        if (tile_ok) {
            const int oh = 2 * ty, ow = 2 * tx;
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int k = ks * 32 + half * 16 + lq * 4 + r;
                    if (k >= P.K) continue;
                    store_tile(y, P.om, P.OH, P.OW, (size_t)n * P.K + k, oh, ow, Y[0][0][half][r], Y[0][1][half][r],
                               Y[1][0][half][r], Y[1][1][half][r]);
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
    if (d.C > 127 || d.nh > 15 || d.nw > 15) return false;
    // classes = pairs of families; inside a class the rows (part, channel) follow each other sorted by
    // (len_h, len_w), longest first, and only the class's end is padded to a multiple of four.  A step
    // whose four rows mix piece lengths runs the planes of the longest: the shorter pieces' rows hold
    // zeros in the filter copy for the frequencies they lack.
    int rows = 0, steps = 0;
    int row_lh[kFusedMaxRows], row_lw[kFusedMaxRows];
    for (int wh = 1; wh >= 0; --wh)
        for (int ww = 1; ww >= 0; --ww) {
            FusedClass fc{};
            fc.wide_h = wh; fc.wide_w = ww;
            fc.nfh = wh ? 4 : 2; fc.nfw = ww ? 4 : 2;
            fc.step0 = steps; fc.row0 = rows;
            for (int lh = 3; lh >= 1; --lh)
                for (int lw = 3; lw >= 1; --lw) {
                    if ((lh >= 2) != (wh == 1) || (lw >= 2) != (ww == 1)) continue;
                    for (int a = 0; a < d.nh; ++a)
                        for (int b = 0; b < d.nw; ++b) {
                            if (d.ph[a].l != lh || d.pw[b].l != lw) continue;
                            for (int c = 0; c < d.C; ++c) {
                                if (rows >= kFusedMaxRows) return false;
                                f.rowdesc[rows] = (unsigned short)(a | b << 4 | c << 8 | 1 << 15);
                                row_lh[rows] = lh; row_lw[rows] = lw;
                                ++rows;
                            }
                        }
                }
            if (rows == fc.row0) continue;
            while ((rows - fc.row0) & 3) {  // padding rows: a real row's offsets, zero filter rows
                if (rows >= kFusedMaxRows) return false;
                f.rowdesc[rows] = (unsigned short)(f.rowdesc[rows - 1] & 0x7fff);
                row_lh[rows] = row_lh[rows - 1]; row_lw[rows] = row_lw[rows - 1];
                ++rows;
            }
            for (int r0 = fc.row0; r0 < rows; r0 += 4) {
                if (steps >= kFusedMaxSteps) return false;
                int mh = 0, mw = 0;
                for (int r = r0; r < r0 + 4; ++r) { mh = std::max(mh, row_lh[r]); mw = std::max(mw, row_lw[r]); }
                f.step_type[steps++] = mh * 4 + mw;
            }
            fc.nsteps = steps - fc.step0;
            fc.rows = rows - fc.row0;
            f.fc[f.nfc++] = fc;
        }
    f.rows_total = rows;

    int max_oh = 0, max_ow = 0;
    for (int i = 0; i < d.nh; ++i) max_oh = std::max(max_oh, d.s * (d.ph[i].j + d.ph[i].l) + d.ph[i].p);
    for (int i = 0; i < d.nw; ++i) max_ow = std::max(max_ow, d.s * (d.pw[i].j + d.pw[i].l) + d.pw[i].p);
    f.nphase = 2 * d.s;
    const size_t table_bytes = (size_t)rows * 64;
    const size_t budget = 72 * 1024;  // two workgroups per CU

    // block of tiles: most useful lanes first, then the smallest staged region
    double best_eff = 0.0;
    size_t best_x = 0;
    for (int bw = 1; bw <= 64 && bw <= d.TW; ++bw) {
        int bh = 64 / bw;
        if (bh > d.TH) bh = d.TH;
        if (bh < 1) continue;
        const int nbh = (d.TH + bh - 1) / bh, nbw = (d.TW + bw - 1) / bw;
        const double eff = (double)d.TH * d.TW / ((double)nbh * nbw * 64);
        const long long nrows = 2LL * d.s * (bh - 1) + max_oh + 1;
        const long long lw_in = 2LL * d.s * (bw - 1) + max_ow + 1;
        const long long lwp = ((lw_in + f.nphase - 1) / f.nphase) | 1;
        const long long x_bytes = (long long)d.C * nrows * f.nphase * lwp * (long long)sizeof(float);
        if (x_bytes + (long long)table_bytes > (long long)budget) continue;
        if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && (size_t)x_bytes < best_x)) {
            best_eff = eff; best_x = (size_t)x_bytes;
            f.BH = bh; f.BW = bw; f.nbh = nbh; f.nbw = nbw;
            f.nrows = (int)nrows; f.lw_in = (int)lw_in; f.lwp = (int)lwp;
        }
    }
    if (best_eff < 0.5) return false;
    const long long blocks = (long long)d.N * f.nbh * f.nbw;
    if (blocks > 0x7fffffffLL) return false;
    f.row_floats = f.nphase * f.lwp;
    f.chan_floats = f.nrows * f.row_floats;
    f.tile_row_step = 2 * d.s * f.row_floats;
    f.nslices = (d.K + 31) / 32;
    // with few blocks the filter slices are spread over workgroups as well
    f.slices_per_wg = blocks >= 2 * kNumCUs ? f.nslices : 1;
    f.nkw = (f.nslices + f.slices_per_wg - 1) / f.slices_per_wg;
    if (f.nkw > 65535) return false;
    f.div_bw.init((unsigned)f.BW);
    f.div_nphase.init((unsigned)f.nphase);
    for (int i = 0; i < kMaxPieces; ++i)
        for (int k = 0; k < 4; ++k) {
            // offsets past a piece's own patch (k > its length) repeat its last element: they are read
            // (the patch is always read 4 wide) and only ever multiplied by zeros, but must be finite
            const int kh = i < d.nh ? std::min(k, d.ph[i].l) : 0, kw = i < d.nw ? std::min(k, d.pw[i].l) : 0;
            const int oh = i < d.nh ? d.s * (d.ph[i].j + kh) + d.ph[i].p : 0;
            const int ow = i < d.nw ? d.s * (d.pw[i].j + kw) + d.pw[i].p : 0;
            f.roff[i][k] = oh * f.row_floats;
            f.coff[i][k] = (ow % f.nphase) * f.lwp + ow / f.nphase;
        }
    f.lds_bytes = table_bytes + best_x;
    *out = f;
    return true;
}

dwm_status_t launch_fused_filter(const dwm_plan& p, const float* w, float* U, void* stream)
{
    if (!p.fused_ok) return DWM_ERR_INVALID_ARG;
    const FusedArgs& f = p.fused;
    dim3 grid((f.rows_total + 255) / 256, f.nslices * 32), block(256);
    hipLaunchKernelGGL(fused_filter_kernel, grid, block, 0, (hipStream_t)stream, p.d, f, w, U, (int)p.uf_gap, (int)p.uf_begin);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

dwm_status_t launch_fused_forward(const dwm_plan& p, const float* x, const float* U, float* y, void* stream)
{
    if (!p.fused_ok) return DWM_ERR_INVALID_ARG;
    const FusedArgs& f = p.fused;
    auto kernel = f.nfc > 1 ? fused_forward_kernel<true> : fused_forward_kernel<false>;
    if (f.lds_bytes > 64 * 1024) {
        // once for each instantiation, whichever of them the first plan happens to use
        static const hipError_t attr = [] {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel<true>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            return hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        }();
        if (attr != hipSuccess) return DWM_ERR_HIP;
    }
    dim3 grid((unsigned)(p.d.N * f.nbh * f.nbw), (unsigned)f.nkw), block(256);
    hipLaunchKernelGGL(kernel, grid, block, f.lds_bytes, (hipStream_t)stream, p.d, f, x, U, y);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

}  // namespace dwm
