// Gradient with respect to the input for layers with few input channels (network stems), in
// one kernel (gfx950).  What is computed is the paper's Sec. 4.2 eq. 16-17 (the parts' input
// gradients summed = the gradient of the ordinary convolution); how:
//
// Pixel (stride*t + rho) of dx, for every residue rho of the pixel coordinate modulo the stride,
// is a sum over ONE window of dy that does not depend on rho (the mirror image of the phase
// grouping of Sec. 4.1, eq. 12-14); only the taps differ.  So all stride^2 phases and all C
// channels of dx are the "filters" f = (c, rho_h, rho_w) of a single stride-1 correlation of dy
// over that window, whose taps are cut into pieces of two and three (eq. 8) that run through
// F(2,2) / F(2,3) (Sec. 3.2).  With C = 3 that gives 12 (stride 2) or 48 (stride 4) columns for
// the matrix unit where a sub-convolution per phase has 3.
//
// A workgroup (four waves) owns a block of tiles of one image and 16 columns; a wave owns 16 tiles.
// The K channels of dy pass through LDS 8, 16 or 32 at a time, double buffered: while a chunk is
// multiplied, the next chunk's region of dy is on its way into registers and its slice of the
// transformed filter into LDS (DMA).  Per step of four reduction rows (four channels of one pair
// of pieces) a lane reads the patch of its (tile, channel) from LDS, applies B^T d B in registers
// -- the result is its B operand for every plane -- and issues one v_mfma_f32_16x16x4_f32 per
// plane; the A operands come from the LDS copy of the filter, four planes per 16-byte read.
// Every plane keeps its own accumulator; A^T M A is applied once at the end, and a lane then
// holds the pixels of its four columns (for stride 2: a 4 x 4 block of one channel), written once.
// dx is fully overwritten (residues no tap reaches have zero filters), nothing is accumulated
// in memory, results do not vary from run to run.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "dma.hpp"
#include "plan.hpp"

namespace dwm {

typedef float bs_float4 __attribute__((ext_vector_type(4)));
typedef float bs_float4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float bs_float2u __attribute__((ext_vector_type(2), aligned(4)));

// (G g)[i] of F(2,3) (Sec. 3.2); a two-tap piece is a three-tap piece whose third tap is zero.
__device__ __forceinline__ float bs_g_row(int i, float v0, float v1, float v2)
{
    switch (i) {
        case 0: return v0;
        case 1: return 0.5f * (v0 + v1 + v2);
        case 2: return 0.5f * (v0 - v1 + v2);
        default: return v2;
    }
}

// ---------------------------------------------------------------------------------
// Filter copy UB[chunk][column block][step][plane, lane]: the A operands exactly as a chunk
// lies in LDS (a chunk padded to whole KB; the padding is copied and never read).  Lane (i, q)
// of a step holds column 16*cb + i and the step's row q; the rows of a chunk are (pair of
// pieces, channel of the chunk).  One thread per (column, channel, pair).
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bwd_small_filter_kernel(BwdSmallArgs F, int R, int S, const float* __restrict__ w,
                                                               float* __restrict__ U)
{
    const int kpad = F.nchunks * F.ck;
    const long long total = (long long)F.ncbp * 16 * kpad * F.npp;  // (blocks that pad the count to whole groups: zeros)
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int pp = (int)(e % F.npp);
    const int k = (int)((e / F.npp) % kpad);
    const int f = (int)(e / ((long long)F.npp * kpad));
    const int ph = pp / F.npw, pw = pp % F.npw;
    const int rho_w = f % F.s, rho_h = (f / F.s) % F.s, c = f / (F.s * F.s);
    const bool real = f < F.nf && k < F.K;
    float g[3][3];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            float v = 0.f;
            if (real && i < F.lh[ph] && j < F.lw[pw]) {
                // window position -> tap of this residue (none: zero)
                const int ih = F.re_h[rho_h] + F.Lh - (F.jh[ph] + i), iw = F.re_w[rho_w] + F.Lw - (F.jw[pw] + j);
                if (ih >= 0 && ih < F.rn_h[rho_h] && iw >= 0 && iw < F.rn_w[rho_w])
                    v = w[(((size_t)k * F.C + c) * R + (F.s * ih + F.ra_h[rho_h])) * S + (F.s * iw + F.ra_w[rho_w])];
            }
            g[i][j] = v;
        }
    float t[4][3];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j) t[i][j] = bs_g_row(i, g[0][j], g[1][j], g[2][j]);
    const int nfreq = F.four ? 4 : 3, planes = nfreq * nfreq;
    const int chunk = k / F.ck, row = pp * F.ck + (k % F.ck);
    const int step = row >> 2, lane = (row & 3) * 16 + (f & 15);
    float* dst = U + ((size_t)chunk * F.ncbp + (f >> 4)) * (size_t)F.us_floats + (size_t)step * (planes * 64);
#pragma unroll
    for (int fh = 0; fh < 4; ++fh)
#pragma unroll
        for (int fw = 0; fw < 4; ++fw)
            if (fh < nfreq && fw < nfreq) dst[bs_upos(planes, fh * nfreq + fw, lane)] = bs_g_row(fw, t[fh][0], t[fh][1], t[fh][2]);
}

// B^T of F(2,3) on a patch of four (Sec. 3.2), or its first three rows on a patch of three
// (two-tap pieces only: the point at infinity is not needed).
template <int NF>
__device__ __forceinline__ void bs_bt(const float (&d)[NF], float (&o)[NF])
{
    o[0] = d[0] - d[2];
    o[1] = d[1] + d[2];
    o[2] = d[2] - d[1];
    if constexpr (NF == 4) o[3] = d[1] - d[3];
}

// A^T over the frequencies of one dimension.
template <int NF>
__device__ __forceinline__ void bs_at(const bs_float4 (&m)[NF], bs_float4 (&o)[2])
{
    o[0] = m[0] + m[1] + m[2];
    o[1] = m[1] - m[2];
    if constexpr (NF == 4) o[1] -= m[3];
}

// NB: blocks of 16 columns a wave keeps accumulators for (one pass over dy serves them all: B^T d B is computed
// once).  Waves per SIMD by the registers that takes: nine planes 3 (NB = 1) or 2; sixteen planes 2 (NB = 1) or 1
// (up to 192 accumulator registers: the MFMAs of one wave, 48 a step, then cover its own vector work).
template <bool FOUR, int NB>
__global__ __launch_bounds__(256, FOUR ? (NB == 1 ? 2 : 1) : (NB == 1 ? 3 : 2)) void bwd_small_kernel(BwdSmallArgs F, const float* __restrict__ dy,
                                                           const float* __restrict__ U, float* __restrict__ dx)
{
    constexpr int NF = FOUR ? 4 : 3, PL = NF * NF, G4 = PL / 4, REM = PL - 4 * G4;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    // LDS: two staged chunks of dy [group of 4 channels][channel pair][row][column parity][lwp][2 channels] | two chunks of
    // the filter copy | per pair of pieces the byte offsets of patch column 0 and 1
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;  // LDS byte address of the array
    const uint32_t xs_bytes = (uint32_t)F.xs_floats * 4u, us_bytes = (uint32_t)F.us_floats * 4u;
    const uint32_t us0 = 2u * xs_bytes, tab0 = us0 + 2u * (uint32_t)NB * us_bytes;  // (a stage holds NB column blocks)
    const char* ldsb = reinterpret_cast<const char*>(lds);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 15, lq = lane >> 4;
    const int tl = wave * 16 + ln;
    const int by = F.div_bw.div(tl), bx = tl - by * F.BW;
    // a lane reads channel lq of a group: plane lq >> 1 of the group, 8 bytes per element, channel lq & 1 of it
    const uint32_t row_bytes = (uint32_t)F.row_elems * 8u, pair_bytes = (uint32_t)F.group_elems * 8u;
    const uint32_t group_bytes = 2u * pair_bytes;
    const uint32_t lane_base = 8u * (uint32_t)(by < F.BH ? by * F.tile_row_step + bx : 0) + 4u * (uint32_t)(lq & 1) +
                               (uint32_t)(lq >> 1) * pair_bytes;
    const size_t img = (size_t)F.OH * F.OW;
    const int region = F.nrows * F.lw_in;
    const int G = 1 << F.glog, NE = 1 << F.nelog;

    if (tid < F.npp) reinterpret_cast<int2*>(lds + (tab0 >> 2))[tid] = make_int2(F.po0[tid], F.po1[tid]);
    // (the first barrier below comes before any wave reads the table)

    const int nblocks = F.N * F.nbh * F.nbw;
    for (int b = blockIdx.x; b < nblocks; b += gridDim.x) {
        const int btx = b % F.nbw, bty = (b / F.nbw) % F.nbh, n = b / (F.nbw * F.nbh);
        const int ty0 = bty * F.BH, tx0 = btx * F.BW;
        const int ty = ty0 + by, tx = tx0 + bx;
        const bool tile_ok = by < F.BH && ty < F.TH && tx < F.TW;

        // What this thread stages of every chunk: slot gs = (group gs >> nelog of the chunk, element
        // tid + 256 * (gs & (NE - 1)) of the block's region of dy), four channels each.  Positions outside the
        // image get an offset past the buffer's end, which reads as zero.
        uint32_t goff[kBsMaxSlots];
        int loff[kBsMaxSlots];
#pragma unroll
        for (int gs = 0; gs < kBsMaxSlots; ++gs) {
            const int idx = tid + 256 * (gs & (NE - 1));
            const int r = F.div_lw.div(idx), c = idx - r * F.lw_in;
            const int row = 2 * ty0 - F.Lh + r, col = 2 * tx0 - F.Lw + c;
            const bool inb = idx < region && row >= 0 && row < F.OH && col >= 0 && col < F.OW;
            goff[gs] = inb ? (uint32_t)(row * F.OW + col) * 4u : 0x80000000u;
            loff[gs] = idx < region && gs < (G << F.nelog)
                           ? (int)((uint32_t)(gs >> F.nelog) * group_bytes) + 8 * (r * F.row_elems + (c & 1) * F.lwp + (c >> 1))
                           : -1;
        }
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(dy + (size_t)n * F.K * img), 0, (int)((size_t)F.K * img * 4), 0x00020000);

        bs_float4 sv[kBsMaxSlots];
        auto stage_load = [&](int chunk) {  // chunk's region of dy -> registers
            const int k0 = chunk * F.ck;
#pragma unroll
            for (int gs = 0; gs < kBsMaxSlots; ++gs) {
                if (gs < (G << F.nelog)) {
                    const int g = gs >> F.nelog;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int k = k0 + 4 * g + j;
                        const uint32_t koff = k < F.K ? 0u : 0x80000000u;  // channels past K: zeros
                        const uint32_t soff = (uint32_t)((size_t)min(k, F.K - 1) * img * 4);
                        sv[gs][j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, goff[gs] | koff, soff, 0));
                    }
                }
            }
        };
        auto stage_write = [&](int buf) {  // registers -> LDS, the two channels of a pair at a time
            char* xb = reinterpret_cast<char*>(lds) + (uint32_t)buf * xs_bytes;
#pragma unroll
            for (int gs = 0; gs < kBsMaxSlots; ++gs)
                if (gs < (G << F.nelog) && loff[gs] >= 0) {
                    *reinterpret_cast<float2*>(xb + (uint32_t)loff[gs]) = make_float2(sv[gs][0], sv[gs][1]);
                    *reinterpret_cast<float2*>(xb + (uint32_t)loff[gs] + pair_bytes) = make_float2(sv[gs][2], sv[gs][3]);
                }
        };

        for (int cb0 = 0; cb0 < F.ncb; cb0 += NB) {
            // a chunk of the filter copy (NB column blocks, adjacent in memory) -> LDS by DMA: 16 bytes per lane,
            // 1 KB per wave and instruction
            auto stage_u = [&](int chunk, int buf) {
                const float* src = U + ((size_t)chunk * F.ncbp + cb0) * F.us_floats;
                const uint32_t dst = lds0 + us0 + (uint32_t)buf * (uint32_t)NB * us_bytes;
                for (uint32_t o = (uint32_t)wave * 1024u; o < (uint32_t)NB * us_bytes; o += 4096u)  // whole KBs
                    dma16s(src, o + (uint32_t)lane * 16u, (uint32_t)__builtin_amdgcn_readfirstlane((int)(dst + o)));
            };

            bs_float4 acc[NB][NF][NF];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < NF; ++i)
#pragma unroll
                    for (int j = 0; j < NF; ++j) acc[nb][i][j] = bs_float4{0.f, 0.f, 0.f, 0.f};

            stage_load(0);
            stage_u(0, 0);
            wait_vmcnt<0>();
            stage_write(0);
            __syncthreads();
            const int2 tab_first = *reinterpret_cast<const int2*>(ldsb + tab0);  // every chunk starts with it

            for (int ci = 0; ci < F.nchunks; ++ci) {
                const int buf = ci & 1;
                const bool more = ci + 1 < F.nchunks;
                if (more) {
                    stage_load(ci + 1);
                    stage_u(ci + 1, buf ^ 1);
                }
                const char* xb = ldsb + (uint32_t)buf * xs_bytes + lane_base;
                const char* ub = ldsb + us0 + (uint32_t)buf * (uint32_t)NB * us_bytes + (uint32_t)lane * 16u;
                const char* ur = ub + (uint32_t)(G4 * 1024) - (uint32_t)lane * 12u;  // (lane * 4 past the 16-byte groups)

                // step st of a chunk = (pair of pieces st >> glog, group st & (G - 1))
                auto read_tab = [&](int st) {
                    return *reinterpret_cast<const int2*>(ldsb + tab0 + (uint32_t)(st >> F.glog) * 8u);
                };
                auto read_patch = [&](int st, int2 t, float (&d)[NF][NF]) {
                    const uint32_t go = (uint32_t)(st & (G - 1)) * group_bytes;
                    const char* p0 = xb + go + (uint32_t)t.x;
                    const char* p1 = xb + go + (uint32_t)t.y;
#pragma unroll
                    for (int i = 0; i < NF; ++i) {
                        const float* q0 = reinterpret_cast<const float*>(p0 + (uint32_t)i * row_bytes);
                        const float* q1 = reinterpret_cast<const float*>(p1 + (uint32_t)i * row_bytes);
                        d[i][0] = q0[0];
                        d[i][2] = q0[2];  // two columns on: the next element of the same parity
                        d[i][1] = q1[0];
                        if constexpr (FOUR) d[i][3] = q1[2];
                    }
                };
                auto read_a = [&](int st, float (&a)[NB][PL]) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const uint32_t so = (uint32_t)nb * us_bytes + (uint32_t)st * (uint32_t)(PL * 256);
#pragma unroll
                        for (int g = 0; g < G4; ++g) {
                            const bs_float4 v = *reinterpret_cast<const bs_float4*>(ub + so + g * 1024);
                            a[nb][4 * g] = v.x; a[nb][4 * g + 1] = v.y; a[nb][4 * g + 2] = v.z; a[nb][4 * g + 3] = v.w;
                        }
#pragma unroll
                        for (int r = 0; r < REM; ++r) a[nb][4 * G4 + r] = *reinterpret_cast<const float*>(ur + so + r * 256);
                    }
                };
                // operands (patch and A) travel a step ahead, the table entries of their pairs of pieces a pass ahead
                auto step = [&](auto next_tag, int st, const float (&d)[NF][NF], float (&dn)[NF][NF], const float (&a)[NB][PL],
                                float (&an)[NB][PL], int2 t) {
                    if constexpr (decltype(next_tag)::value) {
                        read_a(st + 1, an);
                        read_patch(st + 1, t, dn);
                    }
                    float tmp[NF][NF], v[NF][NF];
#pragma unroll
                    for (int j = 0; j < NF; ++j) {
                        float col[NF], o[NF];
#pragma unroll
                        for (int i = 0; i < NF; ++i) col[i] = d[i][j];
                        bs_bt<NF>(col, o);
#pragma unroll
                        for (int i = 0; i < NF; ++i) tmp[i][j] = o[i];
                    }
#pragma unroll
                    for (int i = 0; i < NF; ++i) bs_bt<NF>(tmp[i], v[i]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int i = 0; i < NF; ++i)
#pragma unroll
                            for (int j = 0; j < NF; ++j)
                                acc[nb][i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[nb][i * NF + j], v[i][j], acc[nb][i][j], 0, 0, 0);
                };

                float d0[NF][NF], d1[NF][NF], a0[NB][PL], a1[NB][PL];
                int2 t1 = read_tab(1);
                read_a(0, a0);
                read_patch(0, tab_first, d0);
                int st = 0;
                for (; st + 2 < F.steps; st += 2) {  // steps per chunk: a multiple of two
                    const int2 t2 = read_tab(st + 2), t3 = read_tab(st + 3);
                    step(std::true_type{}, st, d0, d1, a0, a1, t1);
                    step(std::true_type{}, st + 1, d1, d0, a1, a0, t2);
                    t1 = t3;
                }
                step(std::true_type{}, st, d0, d1, a0, a1, t1);
                step(std::false_type{}, st + 1, d1, d0, a1, a0, t1);
                if (more) {
                    wait_vmcnt<0>();
                    stage_write(buf ^ 1);
                }
                __syncthreads();
            }

            // ---- A^T M A, then the lane's pixels: columns 16*cb + 4*lq + r of tile (ty, tx) ----
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
            const int cb = cb0 + nb;
            bs_float4 Y[2][2];
            {
                bs_float4 t[NF][2];
#pragma unroll
                for (int i = 0; i < NF; ++i) bs_at<NF>(acc[nb][i], t[i]);
#pragma unroll
                for (int bcol = 0; bcol < 2; ++bcol) {
                    bs_float4 m[NF], o[2];
#pragma unroll
                    for (int i = 0; i < NF; ++i) m[i] = t[i][bcol];
                    bs_at<NF>(m, o);
                    Y[0][bcol] = o[0];
                    Y[1][bcol] = o[1];
                }
            }
            if (tile_ok && cb < F.ncb) {
                const int f0 = cb * 16 + lq * 4;
                const int s = F.s, ss = s * s;
                float* dxn = dx + (size_t)n * F.C * F.H * F.W;
                if (s == 2) {
                    // the four columns are the four residues of one channel: a 4 x 4 block of pixels
                    const int c = f0 >> 2;
                    if (c < F.C) {
                        float* pc = dxn + (size_t)c * F.H * F.W;
                        const int iw = 4 * tx;
#pragma unroll
                        for (int i = 0; i < 2; ++i)
#pragma unroll
                            for (int rh = 0; rh < 2; ++rh) {
                                const int ih = 4 * ty + 2 * i + rh;
                                if (ih >= F.H) continue;
                                float* pr = pc + (size_t)ih * F.W + iw;
                                const float v0 = Y[i][0][2 * rh], v1 = Y[i][0][2 * rh + 1], v2 = Y[i][1][2 * rh], v3 = Y[i][1][2 * rh + 1];
                                if (iw + 3 < F.W) {
                                    __builtin_nontemporal_store(bs_float4u{v0, v1, v2, v3}, reinterpret_cast<bs_float4u*>(pr));
                                } else {
                                    if (iw < F.W) pr[0] = v0;
                                    if (iw + 1 < F.W) pr[1] = v1;
                                    if (iw + 2 < F.W) pr[2] = v2;
                                }
                            }
                    }
                } else if ((s & 3) == 0) {
                    // the four columns are four adjacent pixels of one row residue
                    const int c = f0 / ss, rh = (f0 / s) % s, rw0 = f0 % s;
                    if (c < F.C) {
                        float* pc = dxn + (size_t)c * F.H * F.W;
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const int ih = s * (2 * ty + i) + rh;
                            if (ih >= F.H) continue;
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                const int iw = s * (2 * tx + j) + rw0;
                                float* pr = pc + (size_t)ih * F.W + iw;
                                if (iw + 3 < F.W) {
                                    __builtin_nontemporal_store(bs_float4u{Y[i][j][0], Y[i][j][1], Y[i][j][2], Y[i][j][3]},
                                                                reinterpret_cast<bs_float4u*>(pr));
                                } else {
                                    if (iw < F.W) pr[0] = Y[i][j][0];
                                    if (iw + 1 < F.W) pr[1] = Y[i][j][1];
                                    if (iw + 2 < F.W) pr[2] = Y[i][j][2];
                                }
                            }
                        }
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int f = f0 + r;
                        if (f >= F.nf) continue;
                        const int c = f / ss, rh = (f / s) % s, rw = f % s;
                        float* pc = dxn + (size_t)c * F.H * F.W;
#pragma unroll
                        for (int i = 0; i < 2; ++i)
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                const int ih = s * (2 * ty + i) + rh, iw = s * (2 * tx + j) + rw;
                                if (ih < F.H && iw < F.W) pc[(size_t)ih * F.W + iw] = Y[i][j][r];
                            }
                    }
                }
            }
            }  // nb
        }
    }
}

dwm_status_t launch_bwd_small_filter(const BwdSmallArgs& a, int R, int S, const float* w, float* U, void* stream)
{
    const long long total = (long long)a.ncbp * 16 * a.nchunks * a.ck * a.npp;
    if (total > 0x7fffffffLL * 256) return DWM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(bwd_small_filter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, a,
                       R, S, w, U);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

dwm_status_t launch_bwd_small(const BwdSmallArgs& a, const float* dy, const float* U, float* dx, void* stream)
{
    using kernel_t = void (*)(BwdSmallArgs, const float*, const float*, float*);
    static const kernel_t kernels[2][3] = {{bwd_small_kernel<false, 1>, bwd_small_kernel<false, 2>, bwd_small_kernel<false, 3>},
                                           {bwd_small_kernel<true, 1>, bwd_small_kernel<true, 2>, bwd_small_kernel<true, 3>}};
    if (a.nb < 1 || a.nb > 3 || a.ncbp % a.nb != 0 || a.ncbp < a.ncb) return DWM_ERR_INVALID_ARG;
    kernel_t kernel = kernels[a.four ? 1 : 0][a.nb - 1];
    if (a.lds_bytes > 64 * 1024) {
        static const hipError_t attr = [] {
            for (int f = 0; f < 2; ++f)
                for (int n = 0; n < 3; ++n) {
                    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernels[f][n]),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
                    if (e != hipSuccess) return e;
                }
            return hipSuccess;
        }();
        if (attr != hipSuccess) return DWM_ERR_HIP;
    }
    // persistent workgroups, as many per CU as registers and LDS allow (fewer where there are fewer blocks)
    const long long nblocks = (long long)a.N * a.nbh * a.nbw;
    const int by_regs = a.four ? (a.nb == 1 ? 2 : 1) : (a.nb == 1 ? 3 : 2);
    const int per_cu = std::max(1, std::min(by_regs, (int)(156 * 1024 / a.lds_bytes)));
    dim3 grid((unsigned)std::min<long long>(nblocks, per_cu * kNumCUs)), block(256);
    hipLaunchKernelGGL(kernel, grid, block, a.lds_bytes, (hipStream_t)stream, a, dy, U, dx);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

}  // namespace dwm
