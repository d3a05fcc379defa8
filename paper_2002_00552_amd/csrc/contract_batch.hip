// Contraction + output transform of SEVERAL stride-1 sub-convolutions in one launch, for the
// gradient with respect to the input (paper Sec. 4.2 eq. 16-17; see backward.hip for how the
// gradient becomes stride^2 sub-convolutions of dy).
//
// Each sub-convolution alone has too few (K tile, T tile) pairs to fill the chip -- the
// stride-2 3x3 layer's four have 196 each on 256 CUs, one workgroup per CU, a fifth of the
// CUs idle -- and they run one after the other on the caller's stream.  Here their tiles form one
// grid, longest sub-convolution first, so that every CU holds two workgroups until the work
// runs out.  A workgroup owns one whole tile of one sub-convolution (no tile is split: the
// grid is several rounds of the CUs deep) and does what the single-problem kernel does:
// operands through a ring of LDS stages filled by global->LDS DMA, one MFMA accumulator folded
// per plane into four running outputs, outputs written through the sub-convolution's output map
// (its phase of dx).
#include <hip/hip_runtime.h>

#include "dma.hpp"
#include "plan.hpp"

namespace dwm {

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int LC, int NS>
__global__ __launch_bounds__(256, 2) void contract_batch_kernel(BatchArgs A, PlaneTable PT,
                                                                const float* __restrict__ U, const float* __restrict__ V,
                                                                float* __restrict__ y)
{
    constexpr int NW = 4, KT = 64, TT = 64;
    constexpr int A_FLOATS = KT * LC, B_FLOATS = LC * TT, STAGE = A_FLOATS + B_FLOATS;
    constexpr int A_I = A_FLOATS / 4 / (64 * NW), B_I = B_FLOATS / 4 / (64 * NW);  // DMA instr. per wave
    constexpr int N_DMA = A_I + B_I;
    constexpr int A_C4 = LC / 4, B_C4 = TT / 4;
    constexpr int GROUPS = LC / 8;
    static_assert(A_I >= 1 && B_I >= 1 && NS >= 2 && (NS - 2) * N_DMA < 64, "LDS ring");

    extern __shared__ __attribute__((aligned(1024))) float smem_b[];  // NS * STAGE floats

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int li = lane & 31, lh = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem_b;

    // which sub-convolution, which of its tiles
    int pi = 0;
    while (pi + 1 < A.nprob && (int)blockIdx.x >= A.p[pi + 1].tile0) ++pi;
    const BatchProb Q = A.p[pi];
    // Workgroups are dealt round-robin to the 8 XCDs: the K tiles of one T tile take launch
    // positions that differ by multiples of 8, so they run on one XCD and share its L2.
    const int r0 = (int)blockIdx.x - Q.tile0;
    const int ntt = (Q.T + TT - 1) / TT, full8 = 8 * A.nkt * (ntt / 8);
    int kt, tt;
    if (r0 < full8) {
        kt = (r0 >> 3) % A.nkt;
        tt = ((r0 >> 3) / A.nkt) * 8 + (r0 & 7);
    } else {
        kt = (r0 - full8) % A.nkt;
        tt = (ntt / 8) * 8 + (r0 - full8) / A.nkt;
    }
    const float* Vp = V + Q.v_base;

    // per-lane source coordinates of this wave's DMA instructions (tile-relative); the XOR
    // patterns are those of the single-problem kernel (conflict-free 16-byte fragment reads)
    auto a_swz = [](int i) {
        if (LC == 16) return ((i >> 1) & 3) ^ ((i >> 3) & 1);
        if (LC == 32) return ((i >> 1) & 7) ^ ((i & 1) << 2);
        return i & 15;
    };
    uint32_t a_row4[A_I], a_col4[A_I];  // 4 * row, 4 * column: byte offset = a_row4 * Lpad + a_col4
    uint32_t b_voff[B_I];               // bytes
#pragma unroll
    for (int q = 0; q < A_I; ++q) {
        const int s = (wave * A_I + q) * 64 + lane;
        const int row = s / A_C4, cp = s % A_C4;
        a_row4[q] = (uint32_t)row * 4u;
        a_col4[q] = (uint32_t)(cp ^ a_swz(row & 31)) * 16u;
    }
#pragma unroll
    for (int q = 0; q < B_I; ++q) {
        const int s = (wave * B_I + q) * 64 + lane;
        const int row = s / B_C4, sp = s % B_C4;
        b_voff[q] = (uint32_t)(row * 64 + (sp ^ (((row >> 2) & 1) << 3)) * 4) * 4u;  // TT = 64: one V block
    }
    const int swz = a_swz(li);

    floatx16 acc, Y[4];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) Y[q][e] = 0.f;

    const int nit = Q.n_iter;
    int p = Q.plane0, j = 0, jf = 0;  // jf: chunks in the accumulator since the last fold
    int nch = PT.e[p].Lpad / LC;

    // issue cursor: the chunk whose loads go out next; parks on the last chunk.  A DMA address is
    // (uniform chunk base) + (the lane's byte offset inside the chunk): moving on is scalar arithmetic.
    int ip = p, ij = 0, inch = nch, ileft = nit;
    const float* sa;
    const float* sb;
    uint32_t ilpad;
    auto point_at = [&](int pl) {
        const DevPlaneEntry e = PT.e[pl];
        sa = U + (size_t)e.u_off64 * 64 + (size_t)(kt * KT) * e.Lpad;
        sb = Vp + (size_t)tt * Q.vblock + (size_t)e.v_off64 * 64;
        ilpad = (uint32_t)e.Lpad;
    };
    point_at(ip);
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
            point_at(ip);
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

        const float* as = smem_b + stage * STAGE + (wave_m * 32 + li) * LC;
        const float* bs = smem_b + stage * STAGE + A_FLOATS + (4 * lh) * TT;
        const int bcol = (wave_n * 32 + li) ^ (lh << 5);
        const int istage = (stage + NS - 1) % NS;
        float4 av[2];
        float bv[2][4];
        auto load_frags = [&](int g, int fb) {
            av[fb] = *reinterpret_cast<const float4*>(as + (((2 * g + lh) ^ swz) * 4));
#pragma unroll
            for (int s = 0; s < 4; ++s) bv[fb][s] = bs[(8 * g + s) * TT + bcol];
        };
        load_frags(0, 0);
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            if (g + 1 < GROUPS) load_frags(g + 1, (g + 1) & 1);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float4 a4 = av[g & 1];
                const float a_s = s == 0 ? a4.x : s == 1 ? a4.y : s == 2 ? a4.z : a4.w;
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_s, bv[g & 1][s], acc, 0, 0, 0);
            }
#pragma unroll
            for (int d = 0; d < N_DMA; ++d)
                if (d * GROUPS / N_DMA == g) issue_one(d, istage);
        }
        advance_issue();

        const bool plane_done = ++j == nch;
        if (plane_done || ++jf == kFoldSteps / LC) {
            jf = 0;
            // fold M_p (or what the accumulator holds of it: long reductions are folded every
            // kFoldSteps steps to keep fp32 partial sums short) into the 2x2 outputs
            const int coef = PT.e[p].coef;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cq = (coef >> (2 * q)) & 3;
                if (cq != 0) {
                    const float sg = cq == 1 ? 1.f : -1.f;
#pragma unroll
                    for (int e = 0; e < 16; ++e) Y[q][e] = fmaf(sg, acc[e], Y[q][e]);
                }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
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
    // every DMA write (the parked re-loads too) has landed before the workgroup ends
    wait_vmcnt<0>();

    // lane holds column t and rows k = 8*(e/4) + 4*lh + e%4 of its 32x32 block
    const int t = tt * TT + wave_n * 32 + li;
    if (t >= Q.T) return;
    const int tiles = Q.TH * Q.TW;
    const int n = t / tiles, rem = t - n * tiles;
    const int ty = rem / Q.TW, tx = rem - ty * Q.TW;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int k = kt * KT + wave_m * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
        if (k >= A.K) continue;
        store_tile(y, Q.om, Q.OH, Q.OW, (size_t)n * A.K + k, 2 * ty, 2 * tx, Y[0][e], Y[1][e], Y[2][e], Y[3][e]);
    }
}

template <int LC, int NS>
static dwm_status_t launch_batch(const BatchArgs& a, const PlaneTable& pt, const float* U, const float* V, float* y,
                                 hipStream_t stream)
{
    constexpr int lds_bytes = NS * (64 + 64) * LC * 4;
    auto kernel = contract_batch_kernel<LC, NS>;
    if (lds_bytes > 64 * 1024) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (attr != hipSuccess) return DWM_ERR_HIP;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)a.ntiles), dim3(256), lds_bytes, stream, a, pt, U, V, y);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

dwm_status_t launch_contract_batch(const BatchArgs& a, const PlaneTable& pt, int lc, const float* U, const float* V,
                                   float* y, void* stream)
{
    switch (lc) {
        case 64: return launch_batch<64, 2>(a, pt, U, V, y, (hipStream_t)stream);
        case 32: return launch_batch<32, 3>(a, pt, U, V, y, (hipStream_t)stream);
        case 16: return launch_batch<16, 4>(a, pt, U, V, y, (hipStream_t)stream);
        default: return DWM_ERR_INVALID_ARG;
    }
}

}  // namespace dwm
