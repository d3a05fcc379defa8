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

// ---------------------------------------------------------------------------------
// Staging of input rows into LDS for the LDS-staged input transforms (single and half
// precision; T is the element type in memory, LDS always holds floats).
// ---------------------------------------------------------------------------------
constexpr int kInLdsBatch = 16;  // input rows a wave loads before it writes them to LDS

// UN consecutive image rows of NC channels, one element per lane each, into consecutive staged
// rows: all NC*UN loads are issued before the first value is used.  xrow: address of the first
// channel's first row, column 0 (the same for the whole wave); voff: the lane's byte offset inside
// a row; channels are chan_bytes apart in memory and chan_floats apart in LDS.
template <int UN, int NC, bool TAIL, typename T>
__device__ __forceinline__ void stage_rows(const char* __restrict__ xrow, unsigned voff, size_t row_bytes,
                                           size_t chan_bytes, float* __restrict__ xd, int row_floats,
                                           int chan_floats, bool iw_ok, int valid)
{
    // TAIL: only the first `valid` (1..UN-1) rows exist; the others re-load the last valid row
    // and are not stored, so that a remainder costs one round of loads instead of one per bit
    T v[NC][UN];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int r = TAIL ? min(u, valid - 1) : u;
            v[c][u] = *reinterpret_cast<const T*>(xrow + c * chan_bytes + r * row_bytes + voff);
        }
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int u = 0; u < UN; ++u)
            if (!TAIL || u < valid) xd[c * chan_floats + u * row_floats] = iw_ok ? (float)v[c][u] : 0.f;
}

// One wave stages NC channels (c, c + cstep, ...) of the input rows that the tiles of a 64-tile
// block touch: the block starts in image n0 at tile row ty_a0 and ends in image n1 at tile row
// ty_b1.  Lanes run along a row, rows go in batches of up to kInLdsBatch loads per channel, image
// by image ("segments", stored one after the other).  Rows above or below the image are written
// as zeros; columns left or right of it are loaded from a clamped (legal) address and replaced by
// zero on the way to LDS.  Columns are de-interleaved modulo 2*stride.  xsc: where channel c goes.
template <typename T, int NC>
__device__ __forceinline__ void stage_channels(const DevPlan& P, const InLdsArgs& A, const T* __restrict__ x,
                                               float* __restrict__ xsc, int c, int cstep, int n0, int n1,
                                               int ty_a0, int ty_b1, int lane)
{
    const int s2 = 2 * P.s;
    const size_t img = (size_t)P.C * P.H * P.W;
    const size_t row_bytes = (size_t)P.W * sizeof(T);
    const size_t chan_bytes = (size_t)cstep * P.H * P.W * sizeof(T);
    const int chan_floats = cstep * A.chan_floats;
    const T* xc = x + ((size_t)n0 * P.C + c) * P.H * P.W;
    for (int cb = 0; cb < A.lw_in; cb += 64) {
        const int col = cb + lane, iw = col - P.Pw;
        const bool iw_ok = iw >= 0 && iw < P.W;
        const unsigned voff = (unsigned)min(max(iw, 0), P.W - 1) * (unsigned)sizeof(T);
        const int idx = A.div_nphase.div(col);
        float* xd = xsc + (col - idx * A.nphase) * A.lwp + idx;
        if (col < A.lw_in) {
            for (int k = 0; k <= n1 - n0; ++k) {
                const int ty_a = k == 0 ? ty_a0 : 0, ty_b = n0 + k == n1 ? ty_b1 : P.TH - 1;
                const int nrows = s2 * (ty_b - ty_a) + A.foot_h, ih0 = s2 * ty_a - P.Ph;
                const int r_lo = min(max(-ih0, 0), nrows), r_hi = max(min(P.H - ih0, nrows), r_lo);
#pragma unroll
                for (int cc = 0; cc < NC; ++cc) {
                    for (int r = 0; r < r_lo; ++r) xd[cc * chan_floats + r * A.row_floats] = 0.f;
                    for (int r = r_hi; r < nrows; ++r) xd[cc * chan_floats + r * A.row_floats] = 0.f;
                }
                const char* xrow = reinterpret_cast<const char*>(xc + (size_t)k * img) + (size_t)(ih0 + r_lo) * row_bytes;
                float* xdr = xd + r_lo * A.row_floats;
                int left = r_hi - r_lo;
                for (; left >= kInLdsBatch; left -= kInLdsBatch) {
                    stage_rows<kInLdsBatch, NC, false, T>(xrow, voff, row_bytes, chan_bytes, xdr, A.row_floats,
                                                          chan_floats, iw_ok, kInLdsBatch);
                    xrow += kInLdsBatch * row_bytes;
                    xdr += kInLdsBatch * A.row_floats;
                }
                if (left > 8)
                    stage_rows<kInLdsBatch, NC, true, T>(xrow, voff, row_bytes, chan_bytes, xdr, A.row_floats,
                                                         chan_floats, iw_ok, left);
                else if (left > 0)
                    stage_rows<8, NC, true, T>(xrow, voff, row_bytes, chan_bytes, xdr, A.row_floats, chan_floats, iw_ok,
                                               left);
                xd += nrows * A.row_floats;
            }
        }
    }
}

}  // namespace dwm
