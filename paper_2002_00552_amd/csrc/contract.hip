// Contraction + output transform + aggregation (paper Sec. 4.1 "Calculation",
// "Detransformation", "Aggregation") for gfx950.
//
// For each plane p = (class, fh, fw):  M_p[k][t] = sum_l U_p[k][l] * V_p[l][t]  -- the
// element-wise product summed over channels, and over the parts of the class because
// A^T(.)A is linear -- is a GEMM on fp32 MFMA.  The output transform is linear too:
//     Y[k][t][a][b] = sum_p AT_lh[a][fh] * AT_lw[b][fw] * M_p[k][t],  coefficients in {0,+1,-1},
// so a workgroup that owns a (K tile, T tile) walks the planes one after the other, keeps
// ONE MFMA accumulator and folds it into four running 2x2 outputs when a plane's
// reduction ends.  M never exists in memory; y is written once.
//
// Data movement: U and V chunks of LC reduction steps go from global memory straight into
// LDS (global_load_lds_dwordx4: 16 bytes per lane, no staging registers, no LDS store
// instructions) through a ring of NS stages: the loads of chunk i+NS-1 are in flight while
// chunk i is multiplied, one barrier per chunk.  LDS rows are unpadded (the DMA writes 64
// consecutive 16-byte slots per wave instruction); bank conflicts are avoided by
// XOR-swizzling which 16-byte column group of a row lands in which slot.
//
// Work distribution: see ContractGeometry.  Tiles left over after the last full round of
// CUs are cut along the iteration axis ("stream-K"); a shared tile is summed, always in
// the same order, by the last workgroup to arrive (no workgroup ever waits for another).
#include <hip/hip_runtime.h>

#include "dma.hpp"
#include "plan.hpp"

namespace dwm {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float pfloat4 __attribute__((ext_vector_type(4)));
typedef unsigned int puint4 __attribute__((ext_vector_type(4)));

struct ContractArgs {
    int K, T, Kpad, Tpad;
    int OH, OW, TH, TW;
    int vblock;  // floats of one 64-tile block of V
    ContractGeometry g;
    OutMap om;   // used by the MAPPED instantiation only
};

// XOR pattern of U-tile row i: which 16-byte column group sits in which slot, chosen so
// that 8 or 16 consecutive lanes reading the same logical group hit distinct banks.
template <int LC>
__device__ __forceinline__ int a_swizzle(int i)
{
    if (LC == 16) return ((i >> 1) & 3) ^ ((i >> 3) & 1);
    if (LC == 32) return ((i >> 1) & 7) ^ ((i & 1) << 2);
    return i & 15;  // LC == 64
}

// MAPPED: outputs go through ContractArgs::om (strided / offset destination, used by the data
// gradient); otherwise y is the dense [N][K][OH][OW] of the forward convolution.
template <int WGM, int WGN, int WM, int WN, int LC, int NS, bool MAPPED>
__global__ __launch_bounds__(64 * WGM * WGN, 8 / (WGM * WGN)) void contract_kernel(
    ContractArgs A, PlaneTable PT, const float* __restrict__ U, const float* __restrict__ V,
    float* __restrict__ y, float* __restrict__ partial, int* __restrict__ counters)
{
    constexpr int NW = WGM * WGN, NT = 64 * NW;
    constexpr int KT = 32 * WM * WGM, TT = 32 * WN * WGN;
    constexpr int A_FLOATS = KT * LC, B_FLOATS = LC * TT, STAGE = A_FLOATS + B_FLOATS;
    constexpr int A_I = A_FLOATS / 4 / (64 * NW), B_I = B_FLOATS / 4 / (64 * NW);  // DMA instr. per wave
    constexpr int N_DMA = A_I + B_I;
    constexpr int A_C4 = LC / 4, B_C4 = TT / 4;
    constexpr int GROUPS = LC / 8;  // groups of 8 reduction steps = 4 MFMA steps
    constexpr int NBLK = WM * WN;
    static_assert(A_I >= 1 && A_I * 256 * NW == A_FLOATS, "U tile must split evenly over the waves");
    static_assert(B_I >= 1 && B_I * 256 * NW == B_FLOATS, "V tile must split evenly over the waves");
    static_assert(TT >= 64 && NS >= 2 && NS * STAGE * 4 <= 160 * 1024, "LDS ring");
    static_assert((NS - 2) * N_DMA < 64, "vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) float smem[];  // NS * STAGE floats
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wave_m = wave / WGN, wave_n = wave % WGN;
    const int li = lane & 31, lh = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    const ContractGeometry& G = A.g;

    // per-lane source coordinates of this wave's DMA instructions (tile-relative)
    uint32_t a_row4[A_I], a_col4[A_I];  // 4 * row, 4 * column: byte offset = a_row4 * Lpad + a_col4
    uint32_t b_voff[B_I];               // bytes
#pragma unroll
    for (int q = 0; q < A_I; ++q) {
        const int s = (wave * A_I + q) * 64 + lane;
        const int row = s / A_C4, cp = s % A_C4;
        a_row4[q] = (uint32_t)row * 4u;
        a_col4[q] = (uint32_t)(cp ^ a_swizzle<LC>(row & 31)) * 16u;
    }
#pragma unroll
    for (int q = 0; q < B_I; ++q) {
        const int s = (wave * B_I + q) * 64 + lane;
        const int row = s / B_C4, sp = s % B_C4;
        const int col = (sp ^ (((row >> 2) & 1) << 3)) * 4;  // column of the V tile this lane fetches
        b_voff[q] = (uint32_t)(row * 64 + (col >> 6) * A.vblock + (col & 63)) * 4u;  // V is blocked by 64 tiles
    }
    const int swz = a_swizzle<LC>(li);

    floatx16 acc[WM][WN];
    floatx16 Y[WM][WN][4];

    // ---- one segment: iterations [it0, it0+nit) of tile (kt, tt); result in Y ----
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
        // plane and chunk of the first iteration; jf: chunks in the accumulator since the last fold
        int p = 0, j = it0, jf = 0;
        int nch = PT.e[0].Lpad / LC;
        while (j >= nch) {
            j -= nch;
            ++p;
            nch = PT.e[p].Lpad / LC;
        }

        // issue cursor: the chunk whose loads go out next; parks on the last chunk of the segment.
        // A DMA address is (uniform chunk base) + (the lane's byte offset inside the chunk): moving to
        // the next chunk is scalar arithmetic, a lane offset changes only with the row length Lpad.
        int ip = p, ij = j, inch = nch, ileft = nit;
        const float* sa;
        const float* sb;
        uint32_t ilpad;  // row length of U in the plane being issued
        auto point_at = [&](int pl, int ch) {
            const DevPlaneEntry e = PT.e[pl];
            sa = U + (size_t)e.u_off64 * 64 + (size_t)(kt * KT) * e.Lpad + ch * LC;
            sb = V + (size_t)(tt * (TT / 64)) * A.vblock + ((size_t)e.v_off64 + ch * LC) * 64;
            ilpad = (uint32_t)e.Lpad;
        };
        point_at(ip, ij);
        auto issue_one = [&](int d, int istage) {
            const uint32_t ls = lds0 + (uint32_t)(istage * STAGE * 4);
            if (d < A_I) dma16s(sa, __umul24(a_row4[d], ilpad) + a_col4[d], ls + (wave * A_I + d) * 1024);
            else dma16s(sb, b_voff[d - A_I], ls + A_FLOATS * 4 + (wave * B_I + (d - A_I)) * 1024);
        };
        auto advance_issue = [&]() {
            if (--ileft <= 0) return;  // parked: the same chunk is loaded again into a free stage
            if (++ij < inch) {
                sa += LC;
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

        // one chunk: multiply what stage holds while the loads of the chunk NS-1 ahead go out
        auto chunk = [&](const int stage, const int it) {
            wait_vmcnt<(NS - 2) * N_DMA>();
            __syncthreads();

            const float* as = smem + stage * STAGE + (wave_m * 32 * WM + li) * LC;
            const float* bs = smem + stage * STAGE + A_FLOATS + (4 * lh) * TT;
            const int bcol = (wave_n * 32 * WN + li) ^ (lh << 5);
            const int istage = (stage + NS - 1) % NS;
            const bool fresh = jf == 0;  // first chunk of a plane, of the segment, or after a fold
            const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            // operand fragments of group g+1 are read from LDS before the MFMAs of group g
            float4 av[2][WM];
            float bv[2][4][WN];
            auto load_frags = [&](int g, int fb) {
#pragma unroll
                for (int mi = 0; mi < WM; ++mi)
                    av[fb][mi] = *reinterpret_cast<const float4*>(as + mi * 32 * LC + (((2 * g + lh) ^ swz) * 4));
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int nj = 0; nj < WN; ++nj) bv[fb][s][nj] = bs[(8 * g + s) * TT + (bcol ^ (nj * 32))];
            };
            load_frags(0, 0);
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                if (g + 1 < GROUPS) load_frags(g + 1, (g + 1) & 1);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
#pragma unroll
                    for (int mi = 0; mi < WM; ++mi) {
                        const float4 a4 = av[g & 1][mi];
                        const float a_s = s == 0 ? a4.x : s == 1 ? a4.y : s == 2 ? a4.z : a4.w;
#pragma unroll
                        for (int nj = 0; nj < WN; ++nj) {
                            if (g == 0 && s == 0 && fresh) {
                                // a plane's first product starts from zero: no accumulator is cleared
                                acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_s, bv[0][0][nj], zero16, 0, 0, 0);
                            } else {
                                acc[mi][nj] =
                                    __builtin_amdgcn_mfma_f32_32x32x2f32(a_s, bv[g & 1][s][nj], acc[mi][nj], 0, 0, 0);
                            }
                        }
                    }
                }
                // the loads of the chunk NS - 1 ahead go out between the first four MFMA groups (all of them in a
                // shallower chunk): spread, so that the waves do not queue at the memory pipeline together, but early,
                // so that a two-stage ring's loads have most of this chunk's time to land before the next barrier
                // waits for them (measured on the 7x7 layer with 256 channels: 0.806 -> 0.776 ms per step)
                constexpr int ISSUE_GROUPS = GROUPS < 4 ? GROUPS : 4;
#pragma unroll
                for (int d = 0; d < N_DMA; ++d)
                    if (d * ISSUE_GROUPS / N_DMA == g) issue_one(d, istage);
            }
            advance_issue();

            const bool plane_done = ++j == nch;
            // Long reductions (several parts of a class, many channels) are folded every kFoldSteps
            // steps: the output transform is linear, so it may be applied to partial sums, and an fp32
            // accumulator that never holds more than a few hundred terms keeps the rounding error at
            // the level of a per-part summation (the accuracy the paper's Table 1 reports).
            if (plane_done || it + 1 == nit || ++jf == kFoldSteps / LC) {
                jf = 0;
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
        // the ring position is a compile-time constant inside the body: LDS addresses of the
        // fragment reads and of the DMA targets are immediates
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

    // ---- scatter Y into y: lane holds column t and rows k = 8*(e/4) + 4*lh + e%4 of each block ----
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
                    if (MAPPED) {
                        store_tile(y, A.om, A.OH, A.OW, (size_t)n * A.K + k, oh, ow, y00, y01, y10, y11);
                        continue;
                    }
                    float* yp = y + (((size_t)n * A.K + k) * A.OH + oh) * A.OW + ow;
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
    };

    // tile index -> (kt, tt): the K tiles of one T tile sit on consecutive slots of ONE XCD
    // (workgroups are dealt round-robin to the 8 XCDs), so they share that XCD's L2
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

    // A whole-tile workgroup is the special case "one range that is exactly one tile".
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
            // Release without a flush of the whole L2.  The partial sums were written with device
            // scope (sc1: the store is complete, i.e. counted off vmcnt, once it has reached the level
            // all XCDs share -- it is what a relaxed device-scope atomic store compiles to); every
            // wave waits for its own stores, the barrier collects the workgroup, and only then one
            // lane bumps the tile's arrival counter with a device-scope atomic.  Atomics on one
            // address are totally ordered, so whoever reads "all others have arrived" does so after
            // every other contributor's stores completed, and its own device-scope loads (below;
            // they do not hit in the local L2) then find them.  The workgroup-scope fences only
            // keep the compiler from moving the accesses across the barriers.
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

// ---------------------------------------------------------------------------------
// Launcher
// ---------------------------------------------------------------------------------
template <int WGM, int WGN, int WM, int WN, int LC, int NS>
static dwm_status_t launch_variant(const dwm_plan& p, const float* U, float* V, float* y, void* stream)
{
    constexpr int KT = 32 * WM * WGM, TT = 32 * WN * WGN;
    static_assert(kKAlign % KT == 0 && kTAlign % TT == 0, "padding must cover the tile");
    ContractArgs a;
    a.K = p.d.K; a.T = p.d.T; a.Kpad = p.d.Kpad; a.Tpad = p.d.Tpad;
    a.OH = p.d.OH; a.OW = p.d.OW; a.TH = p.d.TH; a.TW = p.d.TW;
    a.vblock = p.d.vblock_rows * 64;
    a.g = p.geo;
    // the geometry was computed for exactly this shape of variant
    if (a.g.nkt != (p.d.K + KT - 1) / KT || a.g.ntt != (p.d.T + TT - 1) / TT || p.lgran % LC != 0)
        return DWM_ERR_INVALID_ARG;
    const long long blocks = (long long)a.g.n_full + a.g.sk_wgs;
    constexpr int lds_bytes = NS * (KT + TT) * LC * 4;
    const OutMap& m = p.d.om;
    a.om = m;
    const bool dense = m.sy == 1 && m.sx == 1 && m.oy == 0 && m.ox == 0 && m.YH == p.d.OH && m.YW == p.d.OW;
    auto kd = contract_kernel<WGM, WGN, WM, WN, LC, NS, false>;
    auto km = contract_kernel<WGM, WGN, WM, WN, LC, NS, true>;
    if (lds_bytes > 64 * 1024) {
        static const hipError_t attr_d = hipFuncSetAttribute(reinterpret_cast<const void*>(kd),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        static const hipError_t attr_m = hipFuncSetAttribute(reinterpret_cast<const void*>(km),
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (attr_d != hipSuccess || attr_m != hipSuccess) return DWM_ERR_HIP;
    }
    hipLaunchKernelGGL(dense ? kd : km, dim3((unsigned)blocks), dim3(64 * WGM * WGN), lds_bytes, (hipStream_t)stream,
                       a, p.planes, U, static_cast<const float*>(V), y, p.sk_partial(V), p.sk_counters(V));
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

dwm_status_t launch_contract_output(const dwm_plan& p, const float* U, float* V, float* y, void* stream)
{
    switch (p.geo.variant) {
        case 10: return launch_variant<2, 2, 1, 1, 16, 4>(p, U, V, y, stream);
        case 11: return launch_variant<2, 2, 1, 1, 32, 3>(p, U, V, y, stream);
        case 12: return launch_variant<2, 2, 1, 1, 64, 2>(p, U, V, y, stream);
        case 13: return launch_variant<4, 2, 1, 1, 32, 2>(p, U, V, y, stream);
        case 14: return launch_variant<2, 4, 1, 1, 32, 3>(p, U, V, y, stream);
        case 15: return launch_variant<2, 2, 2, 1, 32, 2>(p, U, V, y, stream);
        case 16: return launch_variant<2, 2, 1, 2, 32, 2>(p, U, V, y, stream);
        case 17: return launch_variant<2, 2, 1, 1, 16, 2>(p, U, V, y, stream);
        case 18: return launch_variant<2, 2, 1, 1, 32, 4>(p, U, V, y, stream);
        case 19: return launch_variant<2, 2, 1, 1, 64, 3>(p, U, V, y, stream);
        default: return DWM_ERR_INVALID_ARG;
    }
}

}  // namespace dwm
