// Half-precision DWM forward convolution for gfx950 (the "DWM FP16" setting of the paper's
// Table 1): x, w and y are IEEE binary16, and so are the transformed filter U = G g G^T and the
// transformed input V = B^T d B (each rounded once, to nearest even); the element-wise
// products summed over channels (Sec. 4.1 "Calculation") run on the FP16 matrix cores with FP32
// accumulation, the output transform and the aggregation of the parts are FP32, and y is
// rounded once at the end.
//
// The decomposition, the row space (class, l) and the plane table are those of the
// single-precision staged path, with the kernel cut exactly as eq. 8 writes it.  What differs is
// the memory layout, because the FP16 MFMA takes EIGHT consecutive reduction indices per lane:
//     U16[plane][l/8][k (Kpad)][l%8]        V16[64-tile block][row/8][tile (64)][row%8]
// so that a lane's operand fragment is one 16-byte word, a wave's global->LDS DMA instruction
// moves 64 such words that are contiguous in memory (1 KB: 64 filters or 64 tiles of one group
// of eight rows), and the 32 lanes of an MFMA operand read 512 contiguous bytes of LDS: no
// padding, no swizzle, no bank conflicts.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>

#include "dma.hpp"
#include "plan.hpp"
#include "xform.hpp"

namespace dwm {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float pfloat4 __attribute__((ext_vector_type(4)));
typedef unsigned int puint4 __attribute__((ext_vector_type(4)));

// The binary16 value nearest to v, ties to even, in ONE rounding (a conversion through float
// would round twice).  |v| is scaled so that binary16's last kept bit has weight one, rounded to
// an integer, and scaled back: the result is a binary16 value and converts exactly.
__device__ __forceinline__ half_t half_from_double(double v)
{
    const double a = fabs(v);
    if (!(a > 0.0) || !(a < 65520.0)) return (half_t)(float)v;  // zero, NaN, overflow to infinity
    int lsb = ilogb(a) - 10;
    if (lsb < -24) lsb = -24;  // subnormal range
    const double r = scalbn(rint(scalbn(a, -lsb)), lsb);
    return (half_t)(float)copysign(r, v);
}

// ---------------------------------------------------------------------------------
// Filter transform (Sec. 4.1 "Transformation", kernel side): one thread per (row, k).
// The arithmetic is FP64 so that U is rounded exactly once.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void filter_transform_f16_kernel(DevPlan P, const half_t* __restrict__ w,
                                                                   half_t* __restrict__ U)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (row >= P.rows_total) return;
    const int qi = find_class(P, row);
    const DevClass q = P.cls[qi];
    const int l = row - q.row0;
    const int th = q.lh + 1, tw = q.lw + 1;

    double u[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) u[i][j] = 0.0;

    if (l < q.L && k < P.K) {
        const int slot = l / P.C, c = l - slot * P.C;
        const int a = slot / q.wn, b = slot - a * q.wn;
        const DevPiece hp = P.ph[q.h0 + a], wp = P.pw[q.w0 + b];
        double g[3][3];
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                double v = 0.0;
                if (i < q.lh && j < q.lw) {
                    const int r = P.s * (hp.j + i) + hp.p, s2 = P.s * (wp.j + j) + wp.p;
                    v = (double)w[(((size_t)k * P.C + c) * P.R + r) * P.S + s2];
                }
                g[i][j] = v;
            }
        double t[4][3];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j) t[i][j] = (i < th) ? g_row<double>(q.lh, i, g[0][j], g[1][j], g[2][j]) : 0.0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                u[i][j] = (i < th && j < tw) ? g_row<double>(q.lw, j, t[i][0], t[i][1], t[i][2]) : 0.0;
    }
    half_t* up = U + (size_t)q.u_off + ((size_t)(l >> 3) * P.Kpad + k) * 8 + (l & 7);
    const size_t plane = (size_t)P.Kpad * q.Lpad;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i < th && j < tw) up[(size_t)(i * tw + j) * plane] = half_from_double(u[i][j]);
}

// ---------------------------------------------------------------------------------
// Input transform (Sec. 4.1 "Splitting" of the input and "Transformation"), gather form.
//
// A thread owns one tile and EIGHT consecutive rows of the flattened (class, l) space -- one
// 16-byte word of every plane of the class.  For each row it gathers the part's patch from
// global memory (binary16 loads; L1/L2 absorb the overlap of neighbouring patches), applies
// B^T . B in FP32 -- exact but for sums that span more than 13 binades -- and rounds to binary16.
// A wave's store is 1 KB contiguous per plane.
// ---------------------------------------------------------------------------------
// pc: the pieces' (phase, offset) in LDS, [dimension][piece][2] -- eight look-ups by a run-time
// index into the by-value plan would make the compiler keep the whole plan in scratch memory
template <int LH, int LW>
__device__ __forceinline__ void input_rows8_f16(const DevPlan& P, const DevClass& q, const int (*pc)[kMaxPieces][2],
                                                const half_t* __restrict__ x, half_t* __restrict__ V, int l0, int t)
{
    constexpr int TH_ = LH + 1, TW_ = LW + 1;
    const bool t_ok = t < P.T;
    const int tiles = P.TH * P.TW;
    const int n = t / tiles, rem = t - n * tiles;
    const int ty = rem / P.TW, tx = rem - ty * P.TW;
    half2_t out[TH_ * TW_][4];
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
        float d[4][TH_][TW_];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int l = l0 + hb * 4 + r;
            const bool row_ok = l < q.L;  // the same for the whole wave: the piece look-ups stay scalar
            const bool ok = row_ok && t_ok;
            const int slot = l / P.C, c = l - slot * P.C;
            const int a = slot / q.wn, b = slot - a * q.wn;
            const int hi = q.h0 + (row_ok ? a : 0), wi = q.w0 + (row_ok ? b : 0);
            const int hp_p = pc[0][hi][0], hp_j = pc[0][hi][1], wp_p = pc[1][wi][0], wp_j = pc[1][wi][1];
            const half_t* xc = x + ((size_t)n * P.C + (row_ok ? c : 0)) * P.H * P.W;
#pragma unroll
            for (int i = 0; i < TH_; ++i) {
                const int ih = P.s * (2 * ty + hp_j + i) + hp_p - P.Ph;
#pragma unroll
                for (int j = 0; j < TW_; ++j) {
                    const int iw = P.s * (2 * tx + wp_j + j) + wp_p - P.Pw;
                    d[r][i][j] =
                        (ok && ih >= 0 && ih < P.H && iw >= 0 && iw < P.W) ? (float)xc[(size_t)ih * P.W + iw] : 0.f;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
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
                for (int j = 0; j < TW_; ++j) out[i * TW_ + j][hb * 2 + (r >> 1)][r & 1] = (half_t)o[j];
            }
        }
    }
    if (!t_ok) return;  // columns past the last tile are never read back into y
    half_t* vp = V + (size_t)(t >> 6) * P.vblock_rows * 64 + ((size_t)((q.v_row0 + l0) >> 3) * 64 + (t & 63)) * 8;
    const size_t plane = (size_t)q.Lpad * 64;
#pragma unroll
    for (int pl = 0; pl < TH_ * TW_; ++pl) {
        uint4 v;
        v.x = __builtin_bit_cast(uint32_t, out[pl][0]);
        v.y = __builtin_bit_cast(uint32_t, out[pl][1]);
        v.z = __builtin_bit_cast(uint32_t, out[pl][2]);
        v.w = __builtin_bit_cast(uint32_t, out[pl][3]);
        *reinterpret_cast<uint4*>(vp + (size_t)pl * plane) = v;
    }
}

__global__ __launch_bounds__(256) void input_transform_f16_kernel(DevPlan P, const half_t* __restrict__ x,
                                                                  half_t* __restrict__ V, int* __restrict__ counters,
                                                                  int n_counters)
{
    // The contraction that follows counts partial-tile arrivals in `counters`; they start at zero.
    if (blockIdx.x == 0 && blockIdx.y == 0)
        for (int i = threadIdx.x; i < n_counters; i += blockDim.x) counters[i] = 0;
    __shared__ int pc[2][kMaxPieces][2];
    if (threadIdx.x < 2 * kMaxPieces) {
        const int i = threadIdx.x % kMaxPieces;
        const DevPiece piece = threadIdx.x < kMaxPieces ? P.ph[i] : P.pw[i];
        pc[threadIdx.x / kMaxPieces][i][0] = piece.p;
        pc[threadIdx.x / kMaxPieces][i][1] = piece.j;
    }
    __syncthreads();
    const int t = blockIdx.x * 64 + (threadIdx.x & 63);  // < Tpad by construction of the grid
    // 8 rows, never across a class (Lpad % 16 == 0); the same for the whole wave, so everything
    // derived from it (class, part, pieces) stays in scalar registers
    const int row = __builtin_amdgcn_readfirstlane((blockIdx.y * 4 + (threadIdx.x >> 6)) * 8);
    if (row >= P.rows_total) return;
    const int qi = find_class(P, row);
    const DevClass q = P.cls[qi];
    const int l0 = row - q.row0;
    switch (q.lh * 4 + q.lw) {
        case 3 * 4 + 3: input_rows8_f16<3, 3>(P, q, pc, x, V, l0, t); break;
        case 3 * 4 + 2: input_rows8_f16<3, 2>(P, q, pc, x, V, l0, t); break;
        case 3 * 4 + 1: input_rows8_f16<3, 1>(P, q, pc, x, V, l0, t); break;
        case 2 * 4 + 3: input_rows8_f16<2, 3>(P, q, pc, x, V, l0, t); break;
        case 2 * 4 + 2: input_rows8_f16<2, 2>(P, q, pc, x, V, l0, t); break;
        case 2 * 4 + 1: input_rows8_f16<2, 1>(P, q, pc, x, V, l0, t); break;
        case 1 * 4 + 3: input_rows8_f16<1, 3>(P, q, pc, x, V, l0, t); break;
        case 1 * 4 + 2: input_rows8_f16<1, 2>(P, q, pc, x, V, l0, t); break;
        default: input_rows8_f16<1, 1>(P, q, pc, x, V, l0, t); break;
    }
}


// ---------------------------------------------------------------------------------
// Input transform, LDS-staged form.
//
// A workgroup owns one 64-tile block of V (lane = tile) and `cg` input channels, a multiple of
// eight.  Its four waves stage the input rows the block's tiles touch (coalesced binary16 loads,
// widened to FP32 on the way to LDS, zero padding written explicitly, columns de-interleaved
// modulo 2*stride so that the same patch element of adjacent tiles sits in adjacent LDS words).
// After one barrier the work items (part, group of eight channels) are dealt to the waves: an
// item reads its eight channels' patches from LDS, transforms them in FP32, rounds, and writes
// one 16-byte word per plane and lane -- 1 KB contiguous per wave store.
// ---------------------------------------------------------------------------------
template <int LH, int LW>
__device__ __forceinline__ void lds_part_rows8(const InLdsArgs& A, const float* __restrict__ xl,
                                               half_t* __restrict__ vp, size_t plane, int hpiece, int wpiece,
                                               bool valid)
{
    constexpr int TH_ = LH + 1, TW_ = LW + 1;
    int ro[TH_], co[TW_];
#pragma unroll
    for (int i = 0; i < TH_; ++i) ro[i] = A.roff[hpiece][i];
#pragma unroll
    for (int j = 0; j < TW_; ++j) co[j] = A.coff[wpiece][j];
    half2_t out[TH_ * TW_][4];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float* xc = xl + c * A.chan_floats;
        float d[TH_][TW_];
#pragma unroll
        for (int i = 0; i < TH_; ++i)
#pragma unroll
            for (int j = 0; j < TW_; ++j) d[i][j] = xc[ro[i] + co[j]];
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
            for (int j = 0; j < TW_; ++j) out[i * TW_ + j][c >> 1][c & 1] = (half_t)o[j];
        }
    }
    if (!valid) return;
#pragma unroll
    for (int pl = 0; pl < TH_ * TW_; ++pl) {
        uint4 v;
        v.x = __builtin_bit_cast(uint32_t, out[pl][0]);
        v.y = __builtin_bit_cast(uint32_t, out[pl][1]);
        v.z = __builtin_bit_cast(uint32_t, out[pl][2]);
        v.w = __builtin_bit_cast(uint32_t, out[pl][3]);
        *reinterpret_cast<uint4*>(vp + (size_t)pl * plane) = v;
    }
}

// The same for ANY channel count: eight consecutive reduction rows l0 .. l0+7 of a class, each with its
// own part (slot = l / C) and channel (l % C) -- wave-uniform values; the pieces' patch offsets come
// from a table in LDS (run-time indexes into the by-value argument struct would put it in scratch);
// rows past the class's reduction length are written as zeros.
template <int LH, int LW>
__device__ __forceinline__ void lds_mixed_rows8(const DevPlan& P, const InLdsArgs& A, const DevClass& q,
                                                const int (*pofs)[kMaxPieces][4], const float* __restrict__ xt,
                                                half_t* __restrict__ vp, size_t plane, int l0, bool valid)
{
    constexpr int TH_ = LH + 1, TW_ = LW + 1;
    half2_t out[TH_ * TW_][4];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int l = l0 + c;
        const bool real = l < q.L;
        const int lc = real ? l : 0;
        const int slot = lc / P.C, ch = lc - slot * P.C;
        const int a = slot / q.wn, bb = slot - a * q.wn;
        const int hpiece = q.h0 + a, wpiece = q.w0 + bb;
        const float* xc = xt + ch * A.chan_floats;
        float d[TH_][TW_];
#pragma unroll
        for (int i = 0; i < TH_; ++i)
#pragma unroll
            for (int j = 0; j < TW_; ++j) d[i][j] = real ? xc[pofs[0][hpiece][i] + pofs[1][wpiece][j]] : 0.f;
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
            for (int j = 0; j < TW_; ++j) out[i * TW_ + j][c >> 1][c & 1] = (half_t)o[j];
        }
    }
    if (!valid) return;
#pragma unroll
    for (int pl = 0; pl < TH_ * TW_; ++pl) {
        uint4 v;
        v.x = __builtin_bit_cast(uint32_t, out[pl][0]);
        v.y = __builtin_bit_cast(uint32_t, out[pl][1]);
        v.z = __builtin_bit_cast(uint32_t, out[pl][2]);
        v.w = __builtin_bit_cast(uint32_t, out[pl][3]);
        *reinterpret_cast<uint4*>(vp + (size_t)pl * plane) = v;
    }
}

__global__ __launch_bounds__(256) void input_transform_f16_lds_kernel(DevPlan P, InLdsArgs A,
                                                                      const half_t* __restrict__ x,
                                                                      half_t* __restrict__ V,
                                                                      int* __restrict__ counters, int n_counters)
{
    extern __shared__ __attribute__((aligned(16))) float xs16[];  // [cg][max_rows][nphase][lwp]
    __shared__ int pofs[2][kMaxPieces][4];  // LDS offsets of the patch rows / columns of every piece
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < n_counters; i += blockDim.x) counters[i] = 0;
    if (threadIdx.x < kMaxPieces * 4) {
        pofs[0][threadIdx.x >> 2][threadIdx.x & 3] = A.roff[threadIdx.x >> 2][threadIdx.x & 3];
        pofs[1][threadIdx.x >> 2][threadIdx.x & 3] = A.coff[threadIdx.x >> 2][threadIdx.x & 3];
    }

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int b = blockIdx.x;
    const int bt = b / A.ncg, bc = b - bt * A.ncg;  // channel groups of one block run together: x rows meet in L2
    const int c0 = bc * A.cg, cn = min(A.cg, P.C - c0);
    const int t0 = bt * 64;
    if (t0 >= P.T) return;  // a block of padding only (Tpad is rounded up to 256)
    const int t1 = min(t0 + 63, P.T - 1);
    const int s2 = 2 * P.s;
    const int g0 = A.div_tw.div(t0), g1 = A.div_tw.div(t1);
    const int n0 = A.div_th.div(g0), n1 = A.div_th.div(g1);
    const int ty_a0 = g0 - n0 * P.TH, ty_b1 = g1 - n1 * P.TH;
    const int rows0 = s2 * ((n1 == n0 ? ty_b1 : P.TH - 1) - ty_a0) + A.foot_h;

    // a wave stages channels wave, wave+4, ...: where cn is a multiple of eight they come in fours or
    // pairs whose loads are in flight together (the staging is a chain of load latencies otherwise)
    int cl = wave;
    for (; cl + 12 < cn; cl += 16)
        stage_channels<half_t, 4>(P, A, x, xs16 + cl * A.chan_floats, c0 + cl, 4, n0, n1, ty_a0, ty_b1, lane);
    for (; cl + 4 < cn; cl += 8)
        stage_channels<half_t, 2>(P, A, x, xs16 + cl * A.chan_floats, c0 + cl, 4, n0, n1, ty_a0, ty_b1, lane);
    for (; cl < cn; cl += 4)  // channel counts that are not a multiple of eight
        stage_channels<half_t, 1>(P, A, x, xs16 + cl * A.chan_floats, c0 + cl, 4, n0, n1, ty_a0, ty_b1, lane);
    __syncthreads();

    const int t = t0 + lane;
    const bool valid = t < P.T;
    int lane_base = 0;
    if (valid) {
        const int g = A.div_tw.div(t), tx = t - g * P.TW;
        const int n = A.div_th.div(g), ty = g - n * P.TH;
        const int base_row = n == n0 ? s2 * (ty - ty_a0) : rows0 + (n - n0 - 1) * A.rows_full + s2 * ty;
        lane_base = base_row * A.row_floats + tx;
    }
    half_t* vb = V + (size_t)bt * P.vblock_rows * 64 + lane * 8;
    if (P.C & 7) {
        // one workgroup holds all channels (cg = C): items are (class, eight rows), padding rows included
        int item = 0;
        for (int qi = 0; qi < P.ncls; ++qi) {
            const DevClass q = P.cls[qi];
            const size_t plane = (size_t)q.Lpad * 64;
            for (int l0 = 0; l0 < q.Lpad; l0 += 8, ++item) {
                if ((item & 3) != wave) continue;
                const float* xt = xs16 + lane_base;
                half_t* vp = vb + (size_t)(q.v_row0 + l0) * 64;
                switch (q.lh * 4 + q.lw) {
                    case 3 * 4 + 3: lds_mixed_rows8<3, 3>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    case 3 * 4 + 2: lds_mixed_rows8<3, 2>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    case 3 * 4 + 1: lds_mixed_rows8<3, 1>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    case 2 * 4 + 3: lds_mixed_rows8<2, 3>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    case 2 * 4 + 2: lds_mixed_rows8<2, 2>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    case 2 * 4 + 1: lds_mixed_rows8<2, 1>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    case 1 * 4 + 3: lds_mixed_rows8<1, 3>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    case 1 * 4 + 2: lds_mixed_rows8<1, 2>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                    default: lds_mixed_rows8<1, 1>(P, A, q, pofs, xt, vp, plane, l0, valid); break;
                }
            }
        }
        return;
    }
    const int ngr = cn >> 3;
    int item = 0;
    for (int qi = 0; qi < P.ncls; ++qi) {
        const DevClass q = P.cls[qi];
        const size_t plane = (size_t)q.Lpad * 64;
        for (int slot = 0; slot < q.hn * q.wn; ++slot)
            for (int g8 = 0; g8 < ngr; ++g8, ++item) {
                if ((item & 3) != wave) continue;
                const int a = slot / q.wn, bb = slot - a * q.wn;
                const float* xl = xs16 + lane_base + g8 * 8 * A.chan_floats;
                half_t* vp = vb + (size_t)(q.v_row0 + slot * P.C + c0 + g8 * 8) * 64;
                const int hp = q.h0 + a, wp = q.w0 + bb;
                switch (q.lh * 4 + q.lw) {
                    case 3 * 4 + 3: lds_part_rows8<3, 3>(A, xl, vp, plane, hp, wp, valid); break;
                    case 3 * 4 + 2: lds_part_rows8<3, 2>(A, xl, vp, plane, hp, wp, valid); break;
                    case 3 * 4 + 1: lds_part_rows8<3, 1>(A, xl, vp, plane, hp, wp, valid); break;
                    case 2 * 4 + 3: lds_part_rows8<2, 3>(A, xl, vp, plane, hp, wp, valid); break;
                    case 2 * 4 + 2: lds_part_rows8<2, 2>(A, xl, vp, plane, hp, wp, valid); break;
                    case 2 * 4 + 1: lds_part_rows8<2, 1>(A, xl, vp, plane, hp, wp, valid); break;
                    case 1 * 4 + 3: lds_part_rows8<1, 3>(A, xl, vp, plane, hp, wp, valid); break;
                    case 1 * 4 + 2: lds_part_rows8<1, 2>(A, xl, vp, plane, hp, wp, valid); break;
                    default: lds_part_rows8<1, 1>(A, xl, vp, plane, hp, wp, valid); break;
                }
            }
        // rows past the class's reduction length are zeros (the contraction multiplies them)
        if (bc == 0 && valid) {
            const int planes = (q.lh + 1) * (q.lw + 1);
            for (int l = q.L + 8 * wave; l < q.Lpad; l += 32)
                for (int pl = 0; pl < planes; ++pl)
                    *reinterpret_cast<uint4*>(vb + (size_t)(q.v_row0 + l) * 64 + (size_t)pl * plane) = make_uint4(0, 0, 0, 0);
        }
    }
}

// ---------------------------------------------------------------------------------
// Contraction + output transform + aggregation (Sec. 4.1 "Calculation", "Detransformation",
// "Aggregation").  Same scheme as the single-precision kernel: a workgroup of WGM x WGN waves owns a
// (K tile, T tile), walks the planes, keeps one MFMA accumulator per 32x32 block and folds it
// with the plane's 0/+-1 pattern into four running 2x2 outputs; operands come through a ring of
// LDS stages filled by global->LDS DMA; leftover tiles are cut along the iteration axis and
// summed in a fixed order by the last workgroup to arrive.
// ---------------------------------------------------------------------------------
struct Contract16Args {
    int K, T, Kpad, Tpad;
    int OH, OW, TH, TW;
    int vblock;  // binary16 elements of one 64-tile block of V
    ContractGeometry g;
};

template <int WGM, int WGN, int WM, int WN, int LC, int NS, bool OUT_F32>
__global__ __launch_bounds__(64 * WGM * WGN, 8 / (WGM * WGN)) void contract16_kernel(Contract16Args A, PlaneTable PT,
                                                            const half_t* __restrict__ U, const half_t* __restrict__ V,
                                                            void* __restrict__ y_out, float* __restrict__ partial,
                                                            int* __restrict__ counters)
{
    constexpr int NW = WGM * WGN, NT = 64 * NW;
    constexpr int KT = 32 * WM * WGM, TT = 32 * WN * WGN;
    constexpr int RG = LC / 8;                               // groups of eight rows per chunk
    constexpr int N_A = RG * (KT / 64), N_B = RG * (TT / 64);  // 1 KB DMA instructions per chunk
    constexpr int N_DMA = (N_A + N_B) / NW;                  // per wave
    constexpr int A_BYTES = KT * LC * 2, B_BYTES = TT * LC * 2, STAGE = A_BYTES + B_BYTES;
    constexpr int STEPS = LC / 16;
    constexpr int NBLK = WM * WN;
    static_assert((N_A + N_B) % NW == 0 && N_DMA >= 1, "DMA instructions must split evenly over the waves");
    static_assert(NS >= 2 && NS * STAGE <= 144 * 1024 && (NS - 2) * N_DMA < 64, "LDS ring");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem16[];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wave_m = wave / WGN, wave_n = wave % WGN;
    const int li = lane & 31, lh = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem16;
    const ContractGeometry& G = A.g;

    // DMA instruction d of this wave is instruction i = d*NW + wave of the chunk; the first N_A
    // fill the U tile [RG][KT][8], the others the V tile [RG][TT][8]: instruction i lands at
    // byte i*1024 of the stage either way.
    // A source address is (uniform base of the chunk in U or V) + (the lane's fixed byte offset).
    bool is_a[N_DMA];
    uint32_t voff[N_DMA];
#pragma unroll
    for (int d = 0; d < N_DMA; ++d) {
        const int i = d * NW + wave;
        is_a[d] = i < N_A;
        if (is_a[d]) {
            const int rg = i / (KT / 64), part = i % (KT / 64);
            voff[d] = (uint32_t)((rg * A.Kpad + part * 64 + lane) * 8) * 2u;
        } else {
            const int rg = (i - N_A) / (TT / 64), blk = (i - N_A) % (TT / 64);
            voff[d] = (uint32_t)(blk * A.vblock + (rg * 64 + lane) * 8) * 2u;
        }
    }

    floatx16 acc[WM][WN];
    floatx16 Y[WM][WN][4];

    auto run_segment = [&](int kt, int tt, int it0, int nit) {
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
        int p = 0, j = it0;
        int nch = PT.e[0].Lpad / LC;
        while (j >= nch) {
            j -= nch;
            ++p;
            nch = PT.e[p].Lpad / LC;
        }

        // issue cursor: the chunk whose loads go out next; parks on the last chunk of the segment
        int ip = p, ij = j, inch = nch, ileft = nit;
        const half_t* sa;
        const half_t* sb;
        auto point_at = [&](int pl, int ch) {
            const DevPlaneEntry e = PT.e[pl];
            sa = U + (size_t)e.u_off64 * 64 + (size_t)ch * LC * A.Kpad + (size_t)(kt * KT) * 8;
            sb = V + (size_t)(tt * (TT / 64)) * A.vblock + ((size_t)e.v_off64 + ch * LC) * 64;
        };
        point_at(ip, ij);
        auto issue_one = [&](int d, int istage) {
            dma16s(reinterpret_cast<const float*>(is_a[d] ? sa : sb), voff[d],
                   lds0 + (uint32_t)(istage * STAGE + (d * NW + wave) * 1024));
        };
        auto advance_issue = [&]() {
            if (--ileft <= 0) return;  // parked: the same chunk is loaded again into a free stage
            if (++ij < inch) {
                sa += (size_t)LC * A.Kpad;
                sb += LC * 64;
            } else {
                ++ip;
                ij = 0;
                inch = PT.e[ip].Lpad / LC;
                point_at(ip, 0);
            }
        };
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) {
#pragma unroll
            for (int d = 0; d < N_DMA; ++d) issue_one(d, s);
            advance_issue();
        }

        auto chunk = [&](const int stage, const int it) {
            wait_vmcnt<(NS - 2) * N_DMA>();
            __syncthreads();

            const unsigned char* as = smem16 + stage * STAGE + (lh * KT + wave_m * 32 * WM + li) * 16;
            const unsigned char* bs = smem16 + stage * STAGE + A_BYTES + (lh * TT + wave_n * 32 * WN + li) * 16;
            const int istage = (stage + NS - 1) % NS;
            const bool fresh = j == 0 || it == 0;  // first chunk of a plane, or of the segment
            const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            half8_t av[2][WM], bv[2][WN];
            auto load_frags = [&](int g, int fb) {
#pragma unroll
                for (int mi = 0; mi < WM; ++mi)
                    av[fb][mi] = *reinterpret_cast<const half8_t*>(as + (2 * g * KT + mi * 32) * 16);
#pragma unroll
                for (int nj = 0; nj < WN; ++nj)
                    bv[fb][nj] = *reinterpret_cast<const half8_t*>(bs + (2 * g * TT + nj * 32) * 16);
            };
            load_frags(0, 0);
#pragma unroll
            for (int g = 0; g < STEPS; ++g) {
                if (g + 1 < STEPS) load_frags(g + 1, (g + 1) & 1);
#pragma unroll
                for (int mi = 0; mi < WM; ++mi)
#pragma unroll
                    for (int nj = 0; nj < WN; ++nj) {
                        if (g == 0 && fresh) {
                            // a plane's first product starts from zero: no accumulator is cleared
                            acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[0][mi], bv[0][nj], zero16, 0, 0, 0);
                        } else {
                            acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[g & 1][mi], bv[g & 1][nj],
                                                                                  acc[mi][nj], 0, 0, 0);
                        }
                    }
                if (g == 0) {
#pragma unroll
                    for (int d = 0; d < N_DMA; ++d) issue_one(d, istage);
                }
            }
            advance_issue();

            const bool plane_done = ++j == nch;
            if (plane_done || it + 1 == nit) {
                // fold M_p (or the part of it this segment covers) into the 2x2 outputs
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
                if (plane_done && it + 1 < nit) {
                    ++p;
                    j = 0;
                    nch = PT.e[p].Lpad / LC;
                }
            }
        };
        // the ring position is a compile-time constant inside the body
        for (int it = 0; it < nit;) {
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                if (it < nit) chunk(st, it);
                ++it;
            }
        }
        // every DMA write (the parked re-loads too) has landed and every wave is done reading
        // before the LDS ring is reused by the next segment or handed to another workgroup
        wait_vmcnt<0>();
        __syncthreads();
    };

    // lane holds column t and rows k = 8*(e/4) + 4*lh + e%4 of each 32x32 block
    auto store_y = [&](int kt, int tt) {
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
                    const float y00 = Y[mi][nj][0][e], y01 = Y[mi][nj][1][e];
                    const float y10 = Y[mi][nj][2][e], y11 = Y[mi][nj][3][e];
                    const size_t idx = (((size_t)n * A.K + k) * A.OH + oh) * A.OW + ow;
                    if (OUT_F32) {
                        float* yp = static_cast<float*>(y_out) + idx;
                        yp[0] = y00;
                        if (ow + 1 < A.OW) yp[1] = y01;
                        if (oh + 1 < A.OH) {
                            yp[A.OW] = y10;
                            if (ow + 1 < A.OW) yp[A.OW + 1] = y11;
                        }
                    } else {
                        half_t* yp = static_cast<half_t*>(y_out) + idx;
                        if (pair_ok) {
                            *reinterpret_cast<half2_t*>(yp) = half2_t{(half_t)y00, (half_t)y01};
                            if (oh + 1 < A.OH) *reinterpret_cast<half2_t*>(yp + A.OW) = half2_t{(half_t)y10, (half_t)y11};
                        } else {
                            yp[0] = (half_t)y00;
                            if (ow + 1 < A.OW) yp[1] = (half_t)y01;
                            if (oh + 1 < A.OH) {
                                yp[A.OW] = (half_t)y10;
                                if (ow + 1 < A.OW) yp[A.OW + 1] = (half_t)y11;
                            }
                        }
                    }
                }
            }
        }
    };

    // tile index -> (kt, tt): the K tiles of one T tile sit on consecutive slots of ONE XCD
    auto tile_coords = [&](int tile, int& kt, int& tt) {
        if (tile < G.full8) {
            const int r0 = tile >> 3;
            kt = r0 % G.nkt;
            tt = (r0 / G.nkt) * 8 + (tile & 7);
        } else {
            const int r0 = tile - G.full8;
            kt = r0 % G.nkt;
            tt = (G.ntt / 8) * 8 + r0 / G.nkt;
        }
    };

    const int b = blockIdx.x;
    const bool whole = b < G.n_full;
    const int gidx = whole ? 0 : b - G.n_full;
    const int tile_base = whole ? b : G.n_full;
    const long long total = (long long)G.n_sk_tiles * G.n_iter;
    long long lo, hi;
    if (whole) {
        lo = 0;
        hi = G.n_iter;
    } else if (G.sk_f > 0) {  // piece gidx % sk_f of tile gidx / sk_f (empty if the tile ran out)
        const long long t0 = (long long)(gidx / G.sk_f) * G.n_iter;
        lo = t0 + (long long)(gidx % G.sk_f) * G.sk_ipw;
        hi = lo + G.sk_ipw < t0 + G.n_iter ? lo + G.sk_ipw : t0 + G.n_iter;
    } else {
        lo = (long long)gidx * G.sk_ipw;
        hi = lo + G.sk_ipw < total ? lo + G.sk_ipw : total;
    }
    constexpr int SLOT = KT * TT * 4;  // floats per partial output
    while (lo < hi) {
        const int trel = (int)(lo / G.n_iter);
        const int it0 = (int)(lo - (long long)trel * G.n_iter);
        const int nit = (int)((G.n_iter - it0 < hi - lo) ? G.n_iter - it0 : hi - lo);
        int kt, tt;
        tile_coords(tile_base + trel, kt, tt);
        run_segment(kt, tt, it0, nit);
        lo += nit;
        bool store = nit == G.n_iter;  // the whole tile was computed here
        if (!store) {
            // contributors of this tile, in iteration order
            const int g_first = G.sk_f > 0 ? trel * G.sk_f : (int)(((long long)trel * G.n_iter) / G.sk_ipw);
            const int g_last = G.sk_f > 0 ? g_first + (G.n_iter - 1) / G.sk_ipw
                                          : (int)((((long long)trel + 1) * G.n_iter - 1) / G.sk_ipw);
            const int nc = g_last - g_first + 1;
            // partial outputs of this tile: [contributor][(block*4 + q)*4 + e/4][thread][4 floats], accessed
            // as a raw buffer with device scope (the accesses complete, or are served, at the
            // level all XCDs share) -- 16-byte accesses that the compiler is free to keep in flight
            // together, which it is not for atomic loads
            const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(
                partial + (size_t)trel * G.sk_maxc * SLOT, 0, (int)((unsigned)G.sk_maxc * SLOT * 4u), 0x00020000);
            constexpr int kDeviceScope = 16;  // cache-policy bits of the access: sc1 = device scope
            const unsigned pvoff = (unsigned)tid * 16u;  // a wave's access is 1 KB contiguous
            const unsigned mine = (unsigned)(gidx - g_first) * (unsigned)(SLOT * 4);
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const floatx16& yv = Y[blk / WN][blk % WN][q];
                        const pfloat4 v = {yv[4 * e4], yv[4 * e4 + 1], yv[4 * e4 + 2], yv[4 * e4 + 3]};
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(puint4, v), prs, pvoff,
                                                               mine + (unsigned)(((blk * 4 + q) * 4 + e4) * NT * 16),
                                                               kDeviceScope);
                    }
            // waiting for the device-scope stores -- not a flush of the whole L2 -- is all the
            // release that the device-scope arrival count below needs (the argument is spelled out at
            // the same place of the single-precision contraction)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            wait_vmcnt<0>();
            __syncthreads();
            if (tid == 0)
                s_last = __hip_atomic_fetch_add(&counters[trel], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nc - 1;
            __syncthreads();
            store = s_last != 0;
            __syncthreads();  // s_last may be rewritten for the next segment
            if (store) {
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                // sum all contributions (this workgroup's own included) in contributor order,
                // so the result does not depend on which workgroup happened to arrive last
                for (int c = 0; c < nc; ++c) {
                    const unsigned soff = (unsigned)c * (unsigned)(SLOT * 4);
#pragma unroll
                    for (int hb = 0; hb < 2 * NBLK; ++hb) {  // half a block (two of its four outputs) at a time
                        pfloat4 v[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            v[i] = __builtin_bit_cast(
                                pfloat4, __builtin_amdgcn_raw_buffer_load_b128(
                                             prs, pvoff, soff + (unsigned)((hb * 8 + i) * NT * 16), kDeviceScope));
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            floatx16& yv = Y[(hb >> 1) / WN][(hb >> 1) % WN][(hb & 1) * 2 + (i >> 2)];
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const float old = yv[4 * (i & 3) + k];
                                yv[4 * (i & 3) + k] = c == 0 ? v[i][k] : old + v[i][k];
                            }
                        }
                    }
                }
                if (tid == 0) counters[trel] = 0;  // ready for the next launch
            }
        }
        if (store) store_y(kt, tt);
    }
}

}  // namespace dwm

// ---------------------------------------------------------------------------------
// Plan and C ABI
// ---------------------------------------------------------------------------------
struct dwm_f16_plan {
    dwm_plan* fwd;  // decomposition, row space, plane table; its geometry is this path's
    unsigned char* ws;
    size_t ws_bytes;
    bool inlds_ok;         // the LDS-staged input transform applies
    dwm::InLdsArgs inlds;
    int variant_input;     // < 0: planner's choice, 0: gather form, 1: LDS-staged form

    static size_t up256(size_t b) { return (b + 255) / 256 * 256; }
    size_t v_bytes() const { return up256(fwd->v_floats * 2); }
    size_t partial_bytes() const { return up256(fwd->geo.partial_floats * sizeof(float)); }
    size_t counters_bytes() const { return up256((size_t)fwd->geo.n_sk_tiles * sizeof(int)); }
    size_t need_bytes() const { return v_bytes() + partial_bytes() + counters_bytes(); }
    dwm::half_t* v() const { return reinterpret_cast<dwm::half_t*>(ws); }
    float* partial() const { return reinterpret_cast<float*>(ws + v_bytes()); }
    int* counters() const { return reinterpret_cast<int*>(ws + v_bytes() + partial_bytes()); }
};

namespace dwm {

// Chunk depth as deep as the layout's row granularity allows; with more than one 64-filter tile
// the workgroup takes 128 filters (eight waves, deeper ring): measured 0.230 -> 0.209 ms on the
// 7x7 layer with 256 channels, equal on the stride-2 3x3 layer.
static int default_variant16(int lgran, int K)
{
    if (lgran >= 64) return K > 64 ? 44 : 32;
    return lgran >= 32 ? 31 : 30;
}

template <int WGM, int WGN, int WM, int WN, int LC, int NS>
static dwm_status_t launch16(const dwm_f16_plan& hp, const half_t* U, void* y, bool out_f32, hipStream_t stream)
{
    const dwm_plan& p = *hp.fwd;
    constexpr int KT = 32 * WM * WGM, TT = 32 * WN * WGN;
    static_assert(kKAlign % KT == 0 && kTAlign % TT == 0, "padding must cover the tile");
    Contract16Args a;
    a.K = p.d.K; a.T = p.d.T; a.Kpad = p.d.Kpad; a.Tpad = p.d.Tpad;
    a.OH = p.d.OH; a.OW = p.d.OW; a.TH = p.d.TH; a.TW = p.d.TW;
    a.vblock = p.d.vblock_rows * 64;
    a.g = p.geo;
    if (a.g.nkt != (p.d.K + KT - 1) / KT || a.g.ntt != (p.d.T + TT - 1) / TT || p.lgran % LC != 0)
        return DWM_ERR_INVALID_ARG;
    const long long blocks = (long long)a.g.n_full + a.g.sk_wgs;
    constexpr int lds_bytes = NS * (KT + TT) * LC * 2;
    auto kh = contract16_kernel<WGM, WGN, WM, WN, LC, NS, false>;
    auto kf = contract16_kernel<WGM, WGN, WM, WN, LC, NS, true>;
    if (lds_bytes + 1024 > 64 * 1024) {  // the kernel has a little static LDS of its own
        static const hipError_t attr_h = hipFuncSetAttribute(reinterpret_cast<const void*>(kh),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        static const hipError_t attr_f = hipFuncSetAttribute(reinterpret_cast<const void*>(kf),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (attr_h != hipSuccess || attr_f != hipSuccess) return DWM_ERR_HIP;
    }
    hipLaunchKernelGGL(out_f32 ? kf : kh, dim3((unsigned)blocks), dim3(64 * WGM * WGN), lds_bytes, stream, a, p.planes, U,
                       hp.v(), y, hp.partial(), hp.counters());
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

static dwm_status_t launch_contract16(const dwm_f16_plan& hp, const half_t* U, void* y, bool out_f32, hipStream_t s)
{
    switch (hp.fwd->geo.variant) {
        case 30: return launch16<2, 2, 1, 1, 16, 4>(hp, U, y, out_f32, s);
        case 31: return launch16<2, 2, 1, 1, 32, 4>(hp, U, y, out_f32, s);
        case 32: return launch16<2, 2, 1, 1, 64, 3>(hp, U, y, out_f32, s);
        case 33: return launch16<2, 2, 1, 2, 32, 3>(hp, U, y, out_f32, s);
        case 34: return launch16<2, 2, 2, 1, 32, 3>(hp, U, y, out_f32, s);
        case 35: return launch16<2, 2, 1, 2, 64, 2>(hp, U, y, out_f32, s);
        case 36: return launch16<4, 2, 1, 1, 64, 2>(hp, U, y, out_f32, s);
        case 37: return launch16<2, 4, 1, 1, 64, 2>(hp, U, y, out_f32, s);
        case 38: return launch16<4, 2, 1, 2, 32, 3>(hp, U, y, out_f32, s);
        case 39: return launch16<2, 4, 2, 1, 32, 3>(hp, U, y, out_f32, s);
        case 40: return launch16<4, 2, 1, 1, 64, 3>(hp, U, y, out_f32, s);
        case 41: return launch16<4, 2, 1, 2, 64, 2>(hp, U, y, out_f32, s);
        case 42: return launch16<2, 2, 1, 1, 64, 5>(hp, U, y, out_f32, s);
        case 43: return launch16<2, 2, 1, 1, 32, 8>(hp, U, y, out_f32, s);
        case 44: return launch16<4, 2, 1, 1, 64, 4>(hp, U, y, out_f32, s);
        case 45: return launch16<4, 2, 1, 2, 64, 3>(hp, U, y, out_f32, s);
        case 46: return launch16<4, 2, 1, 2, 32, 6>(hp, U, y, out_f32, s);
        case 47: return launch16<2, 2, 1, 1, 64, 8>(hp, U, y, out_f32, s);
        default: return DWM_ERR_INVALID_ARG;
    }
}

// The LDS-staged form needs whole groups of eight channels per part and a staged region that
// fits in LDS, preferably with room for three workgroups per CU; with few parts a workgroup takes
// more channels so that each of its four waves has an item.
static bool input16_lds_setup(const dwm_plan& p, InLdsArgs* out)
{
    if (p.d.C % 8 != 0) {
        // all channels in one workgroup, rows in groups of eight across parts and channels
        InLdsArgs a;
        if (p.d.C <= 64 && input_lds_setup(p, &a, p.d.C) && a.cg == p.d.C && a.ncg == 1 && a.lds_bytes <= 48 * 1024) {
            *out = a;
            return true;
        }
        return false;
    }
    const int nparts = p.info.n_parts;
    int cg = 8 * ((4 + nparts - 1) / nparts);
    if (cg > p.d.C) cg = p.d.C;
    InLdsArgs a;
    for (; cg >= 8; cg -= 8)
        if (input_lds_setup(p, &a, cg) && a.cg == cg && a.lds_bytes <= 48 * 1024) {
            *out = a;
            return true;
        }
    // eight channels in a larger region: two workgroups per CU, or one (still far ahead of the
    // gather form, whose 2-byte loads are 2*stride elements apart)
    if (input_lds_setup(p, &a, 8) && a.cg == 8 && a.lds_bytes <= 150 * 1024) {
        *out = a;
        return true;
    }
    return false;
}

static dwm_status_t launch_input16(const dwm_f16_plan& hp, const half_t* x, hipStream_t s)
{
    const DevPlan& d = hp.fwd->d;
    const int nb = d.Tpad / 64, ng = (d.rows_total / 8 + 3) / 4;
    if (hp.variant_input != 0 && hp.inlds_ok) {
        const InLdsArgs& a = hp.inlds;
        if (a.lds_bytes + 1024 > 64 * 1024) {  // the kernel's static table comes on top
            static const hipError_t attr =
                hipFuncSetAttribute(reinterpret_cast<const void*>(input_transform_f16_lds_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 158 * 1024);
            if (attr != hipSuccess) return DWM_ERR_HIP;
        }
        hipLaunchKernelGGL(input_transform_f16_lds_kernel, dim3((unsigned)(nb * a.ncg)), dim3(256), a.lds_bytes, s, d, a,
                           x, hp.v(), hp.counters(), hp.fwd->geo.n_sk_tiles);
        return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
    }
    if (ng > 65535) return DWM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(input_transform_f16_kernel, dim3(nb, ng), dim3(256), 0, s, d, x, hp.v(), hp.counters(),
                       hp.fwd->geo.n_sk_tiles);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

}  // namespace dwm

extern "C" {

dwm_status_t dwm_f16_plan_create(dwm_f16_plan_t** out, int N, int C, int H, int W, int K, int R, int S, int stride,
                                 int pad)
{
    if (!out) return DWM_ERR_INVALID_ARG;
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return DWM_ERR_INVALID_ARG;
    if ((long long)H + 2LL * pad < R || (long long)W + 2LL * pad < S) return DWM_ERR_INVALID_ARG;
    if (pad > (1 << 20) || H > (1 << 20) || W > (1 << 20)) return DWM_ERR_UNSUPPORTED;
    dwm::PlanSpec sp{};
    sp.N = N; sp.C = C; sp.H = H; sp.W = W; sp.K = K; sp.R = R; sp.S = S; sp.stride = stride;
    sp.pad_h = sp.pad_w = pad;
    sp.OH = (H + 2 * pad - R) / stride + 1;
    sp.OW = (W + 2 * pad - S) / stride + 1;
    sp.om = dwm::OutMap{sp.OH, sp.OW, 1, 0, 1, 0};
    dwm_plan_t* fwd = nullptr;
    dwm_status_t st = dwm::plan_from_spec_as_printed(&fwd, sp);
    if (st != DWM_OK) return st;
    if (!dwm::contract_geometry(*fwd, dwm::default_variant16(fwd->lgran, K), &fwd->geo)) {
        dwm_plan_destroy(fwd);
        return DWM_ERR_UNSUPPORTED;
    }
    dwm_f16_plan* hp = new (std::nothrow) dwm_f16_plan;
    if (!hp) {
        dwm_plan_destroy(fwd);
        return DWM_ERR_ALLOC;
    }
    hp->fwd = fwd;
    hp->ws = nullptr;
    hp->ws_bytes = 0;
    hp->variant_input = -1;
    hp->inlds_ok = dwm::input16_lds_setup(*fwd, &hp->inlds);
    *out = hp;
    return DWM_OK;
}

dwm_status_t dwm_f16_plan_destroy(dwm_f16_plan_t* plan)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    dwm_plan_destroy(plan->fwd);
    delete plan;
    return DWM_OK;
}

dwm_status_t dwm_f16_plan_info(const dwm_f16_plan_t* plan, dwm_plan_info_t* info)
{
    if (!plan || !info) return DWM_ERR_INVALID_ARG;
    *info = plan->fwd->info;
    info->forward_path = 0;
    return DWM_OK;
}

size_t dwm_f16_filter_bytes(const dwm_f16_plan_t* plan) { return plan ? plan->fwd->filter_floats * 2 : 0; }
size_t dwm_f16_workspace_bytes(const dwm_f16_plan_t* plan) { return plan ? plan->need_bytes() : 0; }

dwm_status_t dwm_f16_set_workspace(dwm_f16_plan_t* plan, void* ws_dev, size_t bytes)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    if (!ws_dev || ((uintptr_t)ws_dev & 255u) || bytes < plan->need_bytes()) return DWM_ERR_WORKSPACE;
    plan->ws = static_cast<unsigned char*>(ws_dev);
    plan->ws_bytes = bytes;
    return DWM_OK;
}

dwm_status_t dwm_f16_set_variant(dwm_f16_plan_t* plan, const char* stage, int variant)
{
    if (!plan || !stage) return DWM_ERR_INVALID_ARG;
    if (!std::strcmp(stage, "input")) {
        if (variant > 1 || (variant == 1 && !plan->inlds_ok)) return DWM_ERR_INVALID_ARG;
        plan->variant_input = variant;
        return DWM_OK;
    }
    if (std::strcmp(stage, "contract")) return DWM_ERR_INVALID_ARG;
    if (plan->ws) return DWM_ERR_WORKSPACE;  // the variant moves the partial outputs and counters inside the workspace
    if (variant < 0) variant = dwm::default_variant16(plan->fwd->lgran, plan->fwd->d.K);
    if (variant < dwm::kFirstHalfVariant || variant > dwm::kLastHalfVariant) return DWM_ERR_INVALID_ARG;
    dwm::ContractGeometry g;
    if (!dwm::contract_geometry(*plan->fwd, variant, &g)) return DWM_ERR_INVALID_ARG;
    plan->fwd->geo = g;
    return DWM_OK;
}

dwm_status_t dwm_f16_filter_transform(const dwm_f16_plan_t* plan, const dwm_half_t* w_dev, dwm_half_t* U_dev,
                                      void* stream)
{
    if (!plan || !w_dev || !U_dev) return DWM_ERR_INVALID_ARG;
    const dwm::DevPlan& d = plan->fwd->d;
    dim3 grid((d.rows_total + 255) / 256, d.Kpad), block(256);
    hipLaunchKernelGGL(dwm::filter_transform_f16_kernel, grid, block, 0, (hipStream_t)stream, d,
                       reinterpret_cast<const dwm::half_t*>(w_dev), reinterpret_cast<dwm::half_t*>(U_dev));
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

dwm_status_t dwm_f16_input_transform(const dwm_f16_plan_t* plan, const dwm_half_t* x_dev, void* stream)
{
    if (!plan || !x_dev) return DWM_ERR_INVALID_ARG;
    if (!plan->ws) return DWM_ERR_WORKSPACE;
    return dwm::launch_input16(*plan, reinterpret_cast<const dwm::half_t*>(x_dev), (hipStream_t)stream);
}

dwm_status_t dwm_f16_contract_output(const dwm_f16_plan_t* plan, const dwm_half_t* U_dev, dwm_half_t* y_dev,
                                     void* stream)
{
    if (!plan || !U_dev || !y_dev) return DWM_ERR_INVALID_ARG;
    if (!plan->ws) return DWM_ERR_WORKSPACE;
    return dwm::launch_contract16(*plan, reinterpret_cast<const dwm::half_t*>(U_dev), y_dev, false,
                                  (hipStream_t)stream);
}

static dwm_status_t forward16(const dwm_f16_plan_t* plan, const dwm_half_t* x_dev, const dwm_half_t* U_dev,
                              void* y_dev, bool out_f32, void* stream)
{
    if (!plan || !x_dev || !U_dev || !y_dev) return DWM_ERR_INVALID_ARG;
    if (!plan->ws) return DWM_ERR_WORKSPACE;
    const dwm_status_t st = dwm::launch_input16(*plan, reinterpret_cast<const dwm::half_t*>(x_dev), (hipStream_t)stream);
    if (st != DWM_OK) return st;
    return dwm::launch_contract16(*plan, reinterpret_cast<const dwm::half_t*>(U_dev), y_dev, out_f32,
                                  (hipStream_t)stream);
}

dwm_status_t dwm_f16_conv_forward(const dwm_f16_plan_t* plan, const dwm_half_t* x_dev, const dwm_half_t* U_dev,
                                  dwm_half_t* y_dev, void* stream)
{
    return forward16(plan, x_dev, U_dev, y_dev, false, stream);
}

dwm_status_t dwm_f16_conv_forward_f32out(const dwm_f16_plan_t* plan, const dwm_half_t* x_dev, const dwm_half_t* U_dev,
                                         float* y_dev, void* stream)
{
    return forward16(plan, x_dev, U_dev, y_dev, true, stream);
}

}  // extern "C"
