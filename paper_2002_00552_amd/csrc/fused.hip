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
#include <type_traits>

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
template <int WH, int WW, bool ADD>
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
            Y[0][b][half] = ADD ? Y[0][b][half] + o[0] : o[0];
            Y[1][b][half] = ADD ? Y[1][b][half] + o[1] : o[1];
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

// The same from two offsets per patch row: columns 0,2 and 1,3 of a patch are 2*stride input columns
// apart, which is one word in the de-interleaved staged row, so a patch row is two reads of two
// adjacent words (ri: [row][2] offsets of patch rows 0..3 for column 0 and for column 1).
__device__ __forceinline__ void fused_read_patch_pairs(const float* __restrict__ xt, const int4* __restrict__ ri,
                                                       float (&d)[4][4])
{
    const char* xb = reinterpret_cast<const char*>(xt);
    const int4 o0 = ri[0], o1 = ri[1];
    const int a0[4] = {o0.x, o0.y, o0.z, o0.w}, a1[4] = {o1.x, o1.y, o1.z, o1.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float* p0 = reinterpret_cast<const float*>(xb + a0[i]);
        const float* p1 = reinterpret_cast<const float*>(xb + a1[i]);
        d[i][0] = p0[0];
        d[i][2] = p0[1];
        d[i][1] = p1[0];
        d[i][3] = p1[1];
    }
}

// rsrc: raw buffer over the class's filter copy, soff: byte offset of this slice in it; voff = 8 * lane.
// PAIRS: the table holds two offsets per patch row (see above; only with WH = WW = 1), and the
// operands of the class's FIRST step come in through a and d0, fetched by the caller or by the
// previous slice: the last step fetches the first step's operands of the slice at soff_next.  A
// slice's loads are then older than the previous slice's stores to y, so that waiting for them
// (the counter of vector-memory operations runs in issue order) does not wait for those stores.
// ADD: the class's output is added to Y; otherwise it is stored there.
template <int WH, int WW, bool PAIRS, bool ADD>
__device__ __forceinline__ void fused_class(const FusedArgs& F, const FusedClass& fc, const float* __restrict__ xt,
                                         const int4* __restrict__ ri, __amdgpu_buffer_rsrc_t rsrc, unsigned soff,
                                         unsigned soff_next, unsigned voff, float2 (&a)[WH ? 4 : 2][WW ? 4 : 2],
                                         float (&d0)[WH ? 4 : 2][WW ? 4 : 2], floatx4 (&Y)[2][2][2])
{
    constexpr int NH = WH ? 4 : 2, NW = WW ? 4 : 2;
    static_assert(!PAIRS || (WH && WW), "pairs of adjacent words: four-column patches only");
    floatx4 acc[NH][NW][2];  // never cleared: the first step multiplies into zero
    const unsigned plane_bytes = (unsigned)fc.rows * 32u * (unsigned)sizeof(float);
    // A operands travel one step ahead: a plane's registers are refilled for the next step as
    // soon as its MFMAs of this step are issued (the last step refills with itself, or with the next
    // slice's first step).
    float d1[NH][NW];
    auto read_patch = [&](int st, float (&d)[NH][NW]) {
        if constexpr (PAIRS) fused_read_patch_pairs(xt, ri + 8 * st, d);
        else fused_read_patch<NH, NW>(xt, ri + 16 * st, d);
    };
    if (!PAIRS) {
#pragma unroll
        for (int i = 0; i < NH; ++i)
#pragma unroll
            for (int j = 0; j < NW; ++j) a[i][j] = fused_load_a(rsrc, voff, soff + (unsigned)(i * NW + j) * plane_bytes);
        // the patch of the NEXT step is read from LDS before this step's MFMAs are issued; a row's
        // 16 patch offsets (bytes, channel included) come from the table, the lane's tile base is added
        // (two patch buffers that swap roles from step to step: the loop body is written twice)
        read_patch(0, d0);
    }
    int type = F.step_type[fc.step0];
    const floatx4 zero4 = {0.f, 0.f, 0.f, 0.f};
    // one plane of a step: both filter halves; FIRST: the class's first step starts the accumulators
    auto mfma = [&](auto first_tag, int i, int j, float bv, bool on) {
        if constexpr (decltype(first_tag)::value) {
            acc[i][j][0] = on ? __builtin_amdgcn_mfma_f32_16x16x4f32(a[i][j].x, bv, zero4, 0, 0, 0) : zero4;
            acc[i][j][1] = on ? __builtin_amdgcn_mfma_f32_16x16x4f32(a[i][j].y, bv, zero4, 0, 0, 0) : zero4;
        } else {
            if (on) fused_mfma(a[i][j], bv, acc[i][j]);
        }
    };
    auto step = [&](auto first_tag, int st, const float (&d)[NH][NW], float (&dn)[NH][NW]) {
        const bool h3 = !WH || (type >> 2) == 3, w3 = !WW || (type & 3) == 3;  // fourth frequency present
        const bool last = st + 1 >= fc.nsteps;
        const int nst = !last ? st + 1 : PAIRS ? 0 : st;
        type = F.step_type[fc.step0 + nst];
        const unsigned un = (last && PAIRS ? soff_next : soff) + (unsigned)nst * 512u;
        read_patch(nst, dn);
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
                mfma(first_tag, i, j, v[i][j], true);
                a[i][j] = fused_load_a(rsrc, voff, un + (unsigned)(i * NW + j) * plane_bytes);
            }
        if (WW) {
            if (decltype(first_tag)::value || w3) {
#pragma unroll
                for (int i = 0; i < CH; ++i) mfma(first_tag, i, NW - 1, v[i][NW - 1], w3);
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) a[i][NW - 1] = fused_load_a(rsrc, voff, un + (unsigned)(i * NW + 3) * plane_bytes);
        }
        if (WH) {
            if (decltype(first_tag)::value || h3) {
#pragma unroll
                for (int j = 0; j < CW; ++j) mfma(first_tag, NH - 1, j, v[NH - 1][j], h3);
                if (WW) mfma(first_tag, NH - 1, NW - 1, v[NH - 1][NW - 1], h3 && w3);
            }
#pragma unroll
            for (int j = 0; j < NW; ++j) a[NH - 1][j] = fused_load_a(rsrc, voff, un + (unsigned)(3 * NW + j) * plane_bytes);
        }
    };
    step(std::true_type{}, 0, d0, d1);
    int st = 1;
    for (; st + 1 < fc.nsteps; st += 2) {
        step(std::false_type{}, st, d1, d0);
        step(std::false_type{}, st + 1, d0, d1);
    }
    if (st < fc.nsteps) step(std::false_type{}, st, d1, d0);
    if (PAIRS && (fc.nsteps & 1)) {  // the next slice's first patch was read into d1
#pragma unroll
        for (int i = 0; i < NH; ++i)
#pragma unroll
            for (int j = 0; j < NW; ++j) d0[i][j] = d1[i][j];
    }
    fused_output<WH, WW, ADD>(acc, Y);
}

// MULTI: the layer has more than one class, so their outputs are summed in Y; with a single
// class (no one-tap pieces) the registers of Y are saved: the class's output is the result.
// PAIRS (single class of two- and three-tap pieces): patch rows are read as pairs of adjacent words.
template <bool MULTI, bool PAIRS>
__global__ __launch_bounds__(256, 2) void fused_forward_kernel(DevPlan P, FusedArgs F, const float* __restrict__ x,
                                                            const float* __restrict__ U, float* __restrict__ y)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    // LDS: per-row patch offsets | staged input
    constexpr int RI = PAIRS ? 2 : 4;
    int4* rowinfo = reinterpret_cast<int4*>(lds);  // [rows_total][4]: byte offsets [i][j]; PAIRS: [rows_total][2]: [j][i]
    float* xs = reinterpret_cast<float*>(rowinfo + RI * F.rows_total);  // [C][nrows][nphase][lwp]

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 15, lq = lane >> 4;

    // ---- 0. per-row patch offsets (row = part x channel), looked up once ----
    for (int r = tid; r < F.rows_total; r += 256) {
        const unsigned desc = F.rowdesc[r];
        const int base = (int)((desc >> 8) & 127) * F.chan_floats;
        const int* rr = F.roff[desc & 15];
        const int* cc = F.coff[(desc >> 4) & 15];
        if (PAIRS) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
                rowinfo[2 * r + j] = make_int4(4 * (base + rr[0] + cc[j]), 4 * (base + rr[1] + cc[j]),
                                               4 * (base + rr[2] + cc[j]), 4 * (base + rr[3] + cc[j]));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                rowinfo[4 * r + i] = make_int4(4 * (base + rr[i] + cc[0]), 4 * (base + rr[i] + cc[1]),
                                               4 * (base + rr[i] + cc[2]), 4 * (base + rr[i] + cc[3]));
        }
    }

    // Workgroups are persistent: each takes every gridDim.x-th block of tiles (the table above is built
    // once, and a workgroup's last stores need not drain before the CU gets new work).
    const int nblocks = P.N * F.nbh * F.nbw;
    for (int b = blockIdx.x; b < nblocks; b += gridDim.x) {
    if (b != (int)blockIdx.x) __syncthreads();  // every wave is done with the staged input of the block before
    const int btx = b % F.nbw, bty = (b / F.nbw) % F.nbh, n = b / (F.nbw * F.nbh);
    const int ty0 = bty * F.BH, tx0 = btx * F.BW;

    // PAIRS: the first slice's first A operands are asked for before the input is staged (one memory
    // latency instead of two); later slices get theirs from the slice before
    const int slice0 = blockIdx.y * F.slices_per_wg;
    const int slice1 = min(slice0 + F.slices_per_wg, F.nslices);
    const unsigned voff = (unsigned)lane * 8u;
    const FusedClass fc0 = F.fc[0];
    const __amdgpu_buffer_rsrc_t rsrc0 = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(U + fc0.uf_off), 0, (int)((unsigned)(fc0.nfh * fc0.nfw * fc0.rows) * 128u * (unsigned)F.nslices),
        0x00020000);
    float2 a0[4][4];
    if constexpr (PAIRS) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                a0[i][j] = fused_load_a(rsrc0, voff, (unsigned)(slice0 * 16 + i * 4 + j) * ((unsigned)fc0.rows * 128u));
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

    // dense y with an even row length: a uniform base per filter plus the lane's two row offsets
    const int oh = 2 * ty, ow = 2 * tx;
    const bool dense = P.om.sy == 1 && P.om.sx == 1 && P.om.oy == 0 && P.om.ox == 0 && P.om.YH == P.OH &&
                       P.om.YW == P.OW && (P.OW & 1) == 0;
    const unsigned yoff0 = (unsigned)(((lq * 4) * P.OH + oh) * P.OW + ow) * 4u, yoff1 = yoff0 + (unsigned)P.OW * 4u;
    const bool row1 = oh + 1 < P.OH;
    float p0[4][4];
    if constexpr (PAIRS) fused_read_patch_pairs(xt, rowinfo + 2 * lq, p0);
    for (int ks = slice0; ks < slice1; ++ks) {
        floatx4 Y[2][2][2];
        if (MULTI) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int h = 0; h < 2; ++h) Y[a][c][h] = floatx4{0.f, 0.f, 0.f, 0.f};
        }

        if constexpr (PAIRS) {
            const unsigned sbytes = 16u * (unsigned)fc0.rows * 128u;  // one slice of the filter copy
            fused_class<1, 1, true, false>(F, fc0, xt, rowinfo + 2 * lq, rsrc0, (unsigned)ks * sbytes,
                                           (unsigned)(ks + 1 < slice1 ? ks + 1 : ks) * sbytes, voff, a0, p0, Y);
        } else {
            for (int fi = 0; fi < (MULTI ? F.nfc : 1); ++fi) {
                const FusedClass fc = F.fc[fi];
                const unsigned sbytes = (unsigned)(fc.nfh * fc.nfw * fc.rows) * 128u;
                const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<float*>(U + fc.uf_off), 0, (int)(sbytes * (unsigned)F.nslices), 0x00020000);
                const int4* ri = rowinfo + 4 * (fc.row0 + lq);
                const unsigned so = (unsigned)ks * sbytes;
                if (fc.wide_h) {
                    float2 a[4][4];
                    float d[4][4];
                    if (fc.wide_w) fused_class<1, 1, false, MULTI>(F, fc, xt, ri, rsrc, so, so, voff, a, d, Y);
                    else {
                        float2 a2[4][2];
                        float d2[4][2];
                        fused_class<1, 0, false, MULTI>(F, fc, xt, ri, rsrc, so, so, voff, a2, d2, Y);
                    }
                } else {
                    if (fc.wide_w) {
                        float2 a2[2][4];
                        float d2[2][4];
                        fused_class<0, 1, false, MULTI>(F, fc, xt, ri, rsrc, so, so, voff, a2, d2, Y);
                    } else {
                        float2 a2[2][2];
                        float d2[2][2];
                        fused_class<0, 0, false, MULTI>(F, fc, xt, ri, rsrc, so, so, voff, a2, d2, Y);
                    }
                }
            }
        }

        // The next slice's first operands are on their way: they are waited for HERE, before the stores, because
        // the counter of outstanding memory operations runs in issue order -- a wait placed after the stores (whose
        // number depends on the lane's tile and filters, so the compiler cannot count past them) would wait for
        // the stores' round trip as well.
        if constexpr (PAIRS) __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0), nothing else
        // ---- scatter: lane (ln, lq) holds tile ln and filters 32*ks + 16*half + 4*lq + r ----
        if (tile_ok) {
            if (dense) {
#pragma unroll
                for (int half = 0; half < 2; ++half)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int ku = ks * 32 + half * 16 + r;  // + 4*lq is in the lane's offsets
                        if (ku + 4 * lq >= P.K) continue;
                        char* yk = reinterpret_cast<char*>(y + ((size_t)n * P.K + ku) * P.OH * P.OW);
                        // (y is not read again by this kernel: streaming stores)
                        typedef float f2v __attribute__((ext_vector_type(2)));
                        const f2v r0v = {Y[0][0][half][r], Y[0][1][half][r]}, r1v = {Y[1][0][half][r], Y[1][1][half][r]};
                        __builtin_nontemporal_store(r0v, reinterpret_cast<f2v*>(yk + yoff0));
                        if (row1) __builtin_nontemporal_store(r1v, reinterpret_cast<f2v*>(yk + yoff1));
                    }
            } else {
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
    }  // blocks of this workgroup
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
    auto kernel = f.nfc > 1 ? fused_forward_kernel<true, false>
                            : f.wide ? fused_forward_kernel<false, true> : fused_forward_kernel<false, false>;
    if (f.lds_bytes > 64 * 1024) {
        // once for each instantiation, whichever of them the first plan happens to use
        static const hipError_t attr = [] {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel<true, false>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel<false, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            return hipFuncSetAttribute(reinterpret_cast<const void*>(fused_forward_kernel<false, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        }();
        if (attr != hipSuccess) return DWM_ERR_HIP;
    }
    // persistent workgroups, two per CU (fewer where there are fewer blocks)
    const long long nblocks = (long long)p.d.N * f.nbh * f.nbw;
    const long long per_k = std::max<long long>(1, 2 * kNumCUs / f.nkw);
    dim3 grid((unsigned)std::min(nblocks, per_k), (unsigned)f.nkw), block(256);
    hipLaunchKernelGGL(kernel, grid, block, f.lds_bytes, (hipStream_t)stream, p.d, f, x, U, y);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

}  // namespace dwm
