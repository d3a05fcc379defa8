// Gradient of the DWM convolution with respect to its filter (paper Sec. 3.1 eq. 5, second
// formula, and Sec. 4.2 eq. 18): for every part
//     dg = G^T [ sum over tiles and images of (A dY A^T) .* V ] G,      V = B^T d B,
// and a part's dg lands on the taps the part was cut from.
//
// Steps, all on the caller's stream:
//   1. V: the forward pass's input transform of x (same kernel, same layout, blocked by 64 tiles).
//   2. dM = A dY A^T for every plane: the plane's 0/+-1 output pattern applied to the 2x2 block of
//      dy -- the transpose of the forward pass's fold -- written in V's blocked layout,
//      dM[block][plane][k][64 tiles].
//   3. Per plane, dU[k][l] = sum_t dM[k][t] * V[l][t]: a GEMM whose reduction runs over the tiles.
//      fp32 MFMA (32x32x2), 64x64 output tile per workgroup; both operand tiles are "row x 64
//      consecutive tiles", 16 KB contiguous each, brought in by global->LDS DMA with the rows'
//      16-byte groups XOR-swizzled so that the lanes' 16-byte reads do not collide.  The tile
//      axis is cut into `splits` ranges to fill the chip; every range writes its own partial dU.
//   4. The partial dU are summed in a fixed order and G^T (.) G is applied: every tap of dw is
//      written exactly once (the parts partition the taps), nothing is accumulated atomically,
//      results do not vary from run to run.
// Layers with few input channels (every class has at most 32 rows) and many tiles take another
// form of steps 2-3 that never builds dM: see wgrad_small_body / wgrad_small_all_kernel.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>

#include "dma.hpp"
#include "plan.hpp"

namespace dwm {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct WgradArgs {
    int K, Kp, T, tblocks;       // filters, filters rounded up to 64, tiles, blocks of 64 tiles
    int dm_rows, vblock_rows;    // rows of one dM block / one V block
    int n_planes, n_tiles;
    int splits, chunks_per_split;
    long long split_floats;      // floats of one split's partial dU
    int tile0[kMaxPlanes + 1];   // first output tile of each plane
    int nlt[kMaxPlanes];         // 64-wide l tiles of each plane
    int vrow[kMaxPlanes];        // first V row of each plane
    int poff64[kMaxPlanes];      // offset of the plane's dU[Kp][lstride] inside a split, in units of 64 floats
    int lstride[kMaxPlanes];     // floats between consecutive filters k of the plane's dU
};

// ---- step 2: dM[block][plane*Kp + k][t] = sum_q pattern_p[q] * dy[n][k][2ty+a][2tx+b] ----
struct DyShape {
    int T, K, Kp, TH, TW, OH, OW, dm_rows;
};
__global__ __launch_bounds__(256) void wgrad_dy_transform_kernel(DyShape P, PlaneTable PT,
                                                                 const float* __restrict__ dy, float* __restrict__ dM)
{
    const DyShape& A = P;
    const int blk = blockIdx.x;
    const int t = blk * 64 + (threadIdx.x & 63);
    const int k = blockIdx.y * 4 + (threadIdx.x >> 6);
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (t < P.T && k < P.K) {
        const int tiles = P.TH * P.TW;
        const int n = t / tiles, rem = t - n * tiles;
        const int ty = rem / P.TW, tx = rem - ty * P.TW;
        const float* yp = dy + (((size_t)n * P.K + k) * P.OH + 2 * ty) * P.OW + 2 * tx;
        const bool r1 = 2 * ty + 1 < P.OH, c1 = 2 * tx + 1 < P.OW;
        g[0] = yp[0];
        if (c1) g[1] = yp[1];
        if (r1) g[2] = yp[P.OW];
        if (r1 && c1) g[3] = yp[P.OW + 1];
    }
    // rows k >= K and columns t >= T are written as zeros: the GEMM multiplies them
    float* out = dM + ((size_t)blk * A.dm_rows + k) * 64 + (threadIdx.x & 63);
    for (int p = 0; p < PT.n; ++p) {
        const int coef = PT.e[p].coef;
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int cq = (coef >> (2 * q)) & 3;
            v += cq == 1 ? g[q] : cq == 3 ? -g[q] : 0.f;
        }
        out[(size_t)p * A.Kp * 64] = v;
    }
}

// The same with two neighbouring tiles per lane (output rows of a multiple of four pixels: a tile pair's
// two pixel rows are two aligned 16-byte loads, a plane's pair of values one 8-byte store): a wave
// covers two filters x 64 tiles with half the memory instructions.
__global__ __launch_bounds__(256) void wgrad_dy_transform2_kernel(DyShape P, PlaneTable PT,
                                                                  const float* __restrict__ dy, float* __restrict__ dM)
{
    const int blk = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blk * 64 + 2 * (lane & 31);                 // tiles t, t + 1: same tile row (TW is even)
    const int k = blockIdx.y * 8 + wave * 2 + (lane >> 5);
    float4 r0 = make_float4(0.f, 0.f, 0.f, 0.f), r1 = r0;      // pixel rows 2ty, 2ty+1: [t: b=0,1 | t+1: b=0,1]
    if (t < P.T && k < P.K) {
        const int tiles = P.TH * P.TW;
        const int n = t / tiles, rem = t - n * tiles;
        const int ty = rem / P.TW, tx = rem - ty * P.TW;
        const float* yp = dy + (((size_t)n * P.K + k) * P.OH + 2 * ty) * P.OW + 2 * tx;
        r0 = *reinterpret_cast<const float4*>(yp);
        if (2 * ty + 1 < P.OH) r1 = *reinterpret_cast<const float4*>(yp + P.OW);
    }
    const float g0[4] = {r0.x, r0.y, r1.x, r1.y}, g1[4] = {r0.z, r0.w, r1.z, r1.w};
    // rows k >= K and columns t >= T are written as zeros: the GEMM multiplies them
    float* out = dM + ((size_t)blk * P.dm_rows + k) * 64 + 2 * (lane & 31);
    if (k >= P.Kp) return;
    for (int p = 0; p < PT.n; ++p) {
        const int coef = PT.e[p].coef;
        float v0 = 0.f, v1 = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int cq = (coef >> (2 * q)) & 3;
            v0 += cq == 1 ? g0[q] : cq == 3 ? -g0[q] : 0.f;
            v1 += cq == 1 ? g1[q] : cq == 3 ? -g1[q] : 0.f;
        }
        *reinterpret_cast<float2*>(out + (size_t)p * P.Kp * 64) = make_float2(v0, v1);
    }
}

// columns past the last tile of the last V block: zeros (the forward pass leaves them unwritten)
__global__ __launch_bounds__(256) void wgrad_zero_tail_kernel(float* __restrict__ V, int rows, int first_col)
{
    const int ncol = 64 - first_col;
    const size_t total = (size_t)rows * ncol;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256)
        V[(e / ncol) * 64 + first_col + (e % ncol)] = 0.f;
}

// ---- step 3: partial dU of one 64x64 tile of one plane over one range of tile blocks ----
template <int NS>
__global__ __launch_bounds__(256, 2) void wgrad_gemm_kernel(WgradArgs A, const float* __restrict__ dM,
                                                            const float* __restrict__ V, float* __restrict__ partial)
{
    constexpr int TILE = 64 * 64, STAGE = 2 * TILE;  // floats: dM tile + V tile
    constexpr int N_DMA = 8;                         // per wave and chunk: 4 for each tile
    static_assert(NS >= 2 && (NS - 2) * N_DMA < 64, "ring depth");
    extern __shared__ __attribute__((aligned(1024))) float smem[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int li = lane & 31, lh = lane >> 5;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;

    // which tile, which range of blocks
    const int tile = blockIdx.x % A.n_tiles, split = blockIdx.x / A.n_tiles;
    int p = 0;
    while (p + 1 < A.n_planes && tile >= A.tile0[p + 1]) ++p;
    const int r = tile - A.tile0[p];
    const int kt = r / A.nlt[p], lt = r - kt * A.nlt[p];
    const int c0 = split * A.chunks_per_split, c1 = min(c0 + A.chunks_per_split, A.tblocks);
    const int nit = c1 - c0;

    // this wave's DMA sources: rows of 64 floats, 16-byte group cp of row `row` goes to slot cp,
    // fetched from group cp ^ (row & 15).  An address is (uniform chunk base) + (the lane's fixed
    // byte offset): stepping to the next chunk is scalar arithmetic.
    uint32_t voff[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int s = (wave * 4 + q) * 64 + lane;
        const int row = s >> 4, cp = s & 15;
        voff[q] = (uint32_t)(row * 64 + ((cp ^ (row & 15)) << 2)) * 4u;
    }
    const float* sa = dM + ((size_t)c0 * A.dm_rows + (size_t)p * A.Kp + kt * 64) * 64;
    const float* sb = V + ((size_t)c0 * A.vblock_rows + A.vrow[p] + lt * 64) * 64;
    const size_t stepA = (size_t)A.dm_rows * 64, stepB = (size_t)A.vblock_rows * 64;
    int ileft = nit;
    auto issue_chunk = [&](int istage) {
        const uint32_t ls = lds0 + (uint32_t)(istage * STAGE * 4);
#pragma unroll
        for (int q = 0; q < 4; ++q) dma16s(sa, voff[q], ls + (wave * 4 + q) * 1024);
#pragma unroll
        for (int q = 0; q < 4; ++q) dma16s(sb, voff[q], ls + TILE * 4 + (wave * 4 + q) * 1024);
        if (--ileft > 0) {  // the last chunk is simply loaded again: the counts stay uniform
            sa += stepA;
            sb += stepB;
        }
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_chunk(s);

    floatx16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    const int swz = li & 15;
    auto chunk = [&](const int stage) {
        wait_vmcnt<(NS - 2) * N_DMA>();
        __syncthreads();
        // this chunk has landed and every wave is done with the stage the previous one was read
        // from: that stage is refilled while this chunk is multiplied (see the group loop)
        const float* as = smem + stage * STAGE + (wave_m * 32 + li) * 64;
        const float* bs = smem + stage * STAGE + TILE + (wave_n * 32 + li) * 64;
        // the fragments of group g+1 are read from LDS before the MFMAs of group g
        float4 a4[2], b4[2];
        a4[0] = *reinterpret_cast<const float4*>(as + ((lh ^ swz) << 2));
        b4[0] = *reinterpret_cast<const float4*>(bs + ((lh ^ swz) << 2));
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            if (g + 1 < 8) {
                a4[(g + 1) & 1] = *reinterpret_cast<const float4*>(as + (((2 * g + 2 + lh) ^ swz) << 2));
                b4[(g + 1) & 1] = *reinterpret_cast<const float4*>(bs + (((2 * g + 2 + lh) ^ swz) << 2));
                __builtin_amdgcn_sched_barrier(0);  // or the scheduler sinks the reads to their uses
            }
            const float4 a = a4[g & 1], b = b4[g & 1];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
            // the stage the previous chunk was read from is refilled between the first four groups: spread, so
            // that the waves do not queue at the memory pipeline together; early, so that the loads have most of
            // a chunk to land in (measured 1.3 % on the whole filter gradient against all eight at the chunk's start)
            if (g < 4) {
                const uint32_t ls = lds0 + (uint32_t)(((stage + NS - 1) % NS) * STAGE * 4);
                dma16s(sa, voff[g], ls + (wave * 4 + g) * 1024);
                dma16s(sb, voff[g], ls + TILE * 4 + (wave * 4 + g) * 1024);
                if (g == 3 && --ileft > 0) {  // the last chunk is simply loaded again: the counts stay uniform
                    sa += stepA;
                    sb += stepB;
                }
            }
        }
    };
    // the ring position is a compile-time constant inside the body
    for (int it = 0; it < nit;) {
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            if (it < nit) chunk(st);
            ++it;
        }
    }
    wait_vmcnt<0>();

    // lane holds column l = li and rows k = 8*(e/4) + 4*lh + e%4 of its 32x32 block
    const int Lp64 = A.nlt[p] * 64;
    float* out = partial + (size_t)split * A.split_floats + (size_t)A.poff64[p] * 64 +
                 (size_t)(kt * 64 + wave_m * 32) * Lp64 + lt * 64 + wave_n * 32 + li;
#pragma unroll
    for (int e = 0; e < 16; ++e) out[(size_t)(8 * (e >> 2) + 4 * lh + (e & 3)) * Lp64] = acc[e];
}


// ---------------------------------------------------------------------------------
// Short reductions (layers with few input channels: every class has at most 32 rows).
//
// The GEMM form above would multiply 64-row tiles that are mostly padding and, worse, stream
// dM -- planes x K x tiles floats, nine times the size of dy -- through memory twice.  Here a
// workgroup owns 64 filters (16 per wave) and a range of tiles, for ALL planes of one class:
// a lane reads the 2x2 blocks of dy of its filter for four tiles, applies A . A^T in registers
// (the coefficients are compile-time constants), and that is the A operand of
// v_mfma_f32_16x16x4_f32 for every plane; the B operand, V[l][four tiles], is one 16-byte load
// per plane.  Which tile sits in which of the MFMA's four reduction slots is free, so slot q
// of step m takes tile 4q+m: a lane's four steps use exactly its four tiles.  dM never exists.
// Every workgroup writes its own partial dU (compact: [plane][k][Lpad]); a second kernel adds
// the partials in a fixed order.
// ---------------------------------------------------------------------------------
typedef float floatx4 __attribute__((ext_vector_type(4)));

// A^T of F(2,l), row a, column f: the forms of the staged forward path
__host__ __device__ constexpr int at_coef(int l, int a, int f)
{
    return l == 3   ? (a == 0 ? (f < 3 ? 1 : 0) : (f == 0 ? 0 : f == 1 ? 1 : -1))
           : l == 2 ? (a == 0 ? (f < 2 ? 1 : 0) : (f > 0 ? 1 : 0))
                    : (a == f ? 1 : 0);
}

struct SmallArgs {
    int K, Kp, T, OH, OW, TH, TW;
    int vblock_rows, vrow0, Lpad;  // rows of a V block, the class's first row in it, rows per plane
    int L;                         // of which real (the others are zeros, supplied here, not read)
    int r0;                        // first row of a plane this pass covers (a class of more than 32 rows takes two passes)
    int tiles_per_split;           // a multiple of 16
    int poff;                      // floats from the start of a split's partial to this class's planes
    long long split_floats;
    FastDiv div_tiles, div_tw;
};

template <int LH, int LW, int LB>
__device__ __forceinline__ void wgrad_small_body(const SmallArgs& A, const float* __restrict__ dy,
                                                 const float* __restrict__ V, float* __restrict__ partial,
                                                 const int split, const int kt, float (*dys)[16][68],
                                                 float* __restrict__ vs)
{
    constexpr int NH = LH + 1, NW = LW + 1;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int ln = lane & 15, q = lane >> 4;
    const int tiles = A.TH * A.TW;

    floatx4 acc[NH * NW][LB];
#pragma unroll
    for (int p = 0; p < NH * NW; ++p)
#pragma unroll
        for (int lb = 0; lb < LB; ++lb) acc[p][lb] = floatx4{0.f, 0.f, 0.f, 0.f};

    // dy of a chunk of 16 tiles goes through a wave-private piece of LDS so that the global loads
    // are coalesced: for each of the wave's 16 filters one load instruction fetches the two output
    // rows of the 16 tiles (lane = (row a, tile, column b): 128 contiguous bytes per row where the
    // tiles are neighbours); a lane then picks up the 2x2 blocks of ITS filter and four tiles with
    // four 16-byte LDS reads.  Rows are 68 floats apart (64 + 4: conflict-free 16-byte reads).
    float(*my)[68] = dys[wave];
    // V of a chunk -- the class's rows x 16 tiles, the same for the four waves -- is loaded once
    // per workgroup (a thread per (row, 16 bytes)), one chunk ahead, into one of two LDS buffers (vs)
    constexpr int VROWS = NH * NW * LB * 16, VITEMS = (VROWS * 4 + 255) / 256;
    floatx4 vreg[VITEMS];
    // this thread's (row, 16 bytes) items: offsets inside the class's rows of a V block / an LDS buffer
    int vsrc[VITEMS], vdst[VITEMS];
    bool vreal[VITEMS];  // rows past the class's reduction length are not in memory: zeros
#pragma unroll
    for (int it = 0; it < VITEMS; ++it) {
        const int idx = min((int)threadIdx.x + 256 * it, VROWS * 4 - 1);  // spare threads repeat the last item
        const int row = idx >> 2, pl = row / (16 * LB), r = A.r0 + row - pl * (16 * LB);  // plane, row of the plane
        vsrc[it] = (pl * A.Lpad + r) * 64 + 4 * (idx & 3);
        vdst[it] = idx * 4;
        vreal[it] = r < A.L;
    }
#define DWM_LOAD_V(t0_)                                                                                     \
    {                                                                                                       \
        const float* vbase_ = V + ((size_t)((t0_) >> 6) * A.vblock_rows + A.vrow0) * 64 + ((t0_) & 63);       \
        _Pragma("unroll") for (int it = 0; it < VITEMS; ++it)                                               \
            vreg[it] = vreal[it] ? *reinterpret_cast<const floatx4*>(vbase_ + vsrc[it])                      \
                                 : floatx4{0.f, 0.f, 0.f, 0.f};                                              \
    }
#define DWM_STORE_V(buf_)                                                                                   \
    {                                                                                                       \
        _Pragma("unroll") for (int it = 0; it < VITEMS; ++it)                                               \
            *reinterpret_cast<floatx4*>(vs + (buf_) * (VROWS * 16) + vdst[it]) = vreg[it];                    \
    }
    const int la = lane >> 5, lt = (lane >> 1) & 15, lb_ = lane & 1;
    const int kw = kt * 64 + wave * 16;

    const int t_begin = split * A.tiles_per_split;
    const int t_end = min(t_begin + A.tiles_per_split, (A.T + 15) & ~15);
    const size_t kstep = (size_t)A.OH * A.OW;
    float v[16];
    auto load_dy = [&](int t0) {
        const int t = t0 + lt;
        const int n = A.div_tiles.div(min(t, A.T - 1)), rem = min(t, A.T - 1) - n * tiles;
        const int ty = A.div_tw.div(rem), tx = rem - ty * A.TW;
        const bool ok = t < A.T && 2 * ty + la < A.OH && 2 * tx + lb_ < A.OW;
        const float* yp = dy + (((size_t)n * A.K + kw) * A.OH + 2 * ty + la) * A.OW + 2 * tx + lb_;
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = (ok && kw + j < A.K) ? yp[(size_t)j * kstep] : 0.f;
    };
    if (t_begin < t_end) {
        load_dy(t_begin);
        DWM_LOAD_V(t_begin)
    }
    int cur = 0;
    for (int t0 = t_begin; t0 < t_end; t0 += 16, cur ^= 1) {
        DWM_STORE_V(cur)
        __syncthreads();  // also: every wave is done with the other buffer, which the next chunk refills
        if (t0 + 16 < t_end) DWM_LOAD_V(t0 + 16)
        {
            // other lanes of this wave read what this lane writes, and the other way round: the
            // hardware runs a wave's LDS instructions in order; these keep the compiler from
            // moving the reads of one phase across the writes of the other (no instruction emitted)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < 16; ++j) my[j][lane] = v[j];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // the next chunk's dy is in flight while this one is multiplied
            if (t0 + 16 < t_end) load_dy(t0 + 16);
        }
        // r[i][fh][b] = sum_a A^T[a][fh] * dy[a][b] of this lane's tile 4q+i
        float r[4][NH][2];
        {
            const float4 g0 = *reinterpret_cast<const float4*>(&my[ln][8 * q]);
            const float4 g1 = *reinterpret_cast<const float4*>(&my[ln][8 * q + 4]);
            const float4 h0 = *reinterpret_cast<const float4*>(&my[ln][32 + 8 * q]);
            const float4 h1 = *reinterpret_cast<const float4*>(&my[ln][32 + 8 * q + 4]);
            const float g[4][2][2] = {{{g0.x, g0.y}, {h0.x, h0.y}}, {{g0.z, g0.w}, {h0.z, h0.w}},
                                      {{g1.x, g1.y}, {h1.x, h1.y}}, {{g1.z, g1.w}, {h1.z, h1.w}}};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int fh = 0; fh < NH; ++fh)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        r[i][fh][b] = (float)at_coef(LH, 0, fh) * g[i][0][b] + (float)at_coef(LH, 1, fh) * g[i][1][b];
        }
        // B operands: V[row = plane*Lpad + lb*16 + ln][tiles 4q .. 4q+3] of the chunk, from LDS
        const float* vl = vs + cur * (VROWS * 16) + ln * 16 + 4 * q;
#pragma unroll
        for (int p = 0; p < NH * NW; ++p) {
            const int fh = p / NW, fw = p % NW;
            float a[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                a[i] = (float)at_coef(LW, 0, fw) * r[i][fh][0] + (float)at_coef(LW, 1, fw) * r[i][fh][1];
#pragma unroll
            for (int lb = 0; lb < LB; ++lb) {
                const float4 b4 = *reinterpret_cast<const float4*>(vl + (p * LB + lb) * 256);
                acc[p][lb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b4.x, acc[p][lb], 0, 0, 0);
                acc[p][lb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b4.y, acc[p][lb], 0, 0, 0);
                acc[p][lb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b4.z, acc[p][lb], 0, 0, 0);
                acc[p][lb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b4.w, acc[p][lb], 0, 0, 0);
            }
        }
    }
    // lane (ln, q) holds dU[k = 4q + e][l = ln] of its wave's 16 filters
    float* out = partial + (size_t)split * A.split_floats + A.poff +
                 ((size_t)(kt * 64 + wave * 16 + 4 * q)) * A.Lpad + A.r0 + ln;
#pragma unroll
    for (int p = 0; p < NH * NW; ++p)
#pragma unroll
        for (int lb = 0; lb < LB; ++lb)
#pragma unroll
            for (int e = 0; e < 4; ++e) out[((size_t)p * A.Kp + e) * A.Lpad + lb * 16] = acc[p][lb][e];
}

#undef DWM_LOAD_V
#undef DWM_STORE_V

// All classes (of one LB) in ONE launch.  The classes of one (range of tiles, 64 filters) read the
// same dy: their workgroups sit next to each other in launch order on one XCD (launch position
// mod 8), so that dy comes from memory once and from that XCD's L2 for the other classes --
// launched class by class, each class streamed all of dy from memory again.
struct SmallAllArgs {
    int ncls, nkt, splits;
    int code[kMaxClasses];  // 4 * len_h + len_w
    SmallArgs c[kMaxClasses];
};

template <int LB>
__global__ __launch_bounds__(256, 2) void wgrad_small_all_kernel(SmallAllArgs AA, const float* __restrict__ dy,
                                                                 const float* __restrict__ V,
                                                                 float* __restrict__ partial)
{
    __shared__ __attribute__((aligned(16))) float dys[4][16][68];
    extern __shared__ __attribute__((aligned(16))) float vs[];
    // launch position -> (range of tiles, 64 filters, class): class fastest among the groups of eight
    const int b = blockIdx.x, s_lo = b & 7;
    int r = b >> 3;
    const int ci = r % AA.ncls;
    r /= AA.ncls;
    const int kt = r % AA.nkt;
    const int split = (r / AA.nkt) * 8 + s_lo;
    if (split >= AA.splits) return;
    // the class's arguments through compile-time indexes (they stay in scalar registers)
    SmallArgs A = AA.c[0];
    int code = AA.code[0];
#pragma unroll
    for (int i = 1; i < kMaxClasses; ++i)
        if (ci == i) {
            A = AA.c[i];
            code = AA.code[i];
        }
    switch (code) {
        case 3 * 4 + 3: wgrad_small_body<3, 3, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        case 3 * 4 + 2: wgrad_small_body<3, 2, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        case 3 * 4 + 1: wgrad_small_body<3, 1, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        case 2 * 4 + 3: wgrad_small_body<2, 3, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        case 2 * 4 + 2: wgrad_small_body<2, 2, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        case 2 * 4 + 1: wgrad_small_body<2, 1, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        case 1 * 4 + 3: wgrad_small_body<1, 3, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        case 1 * 4 + 2: wgrad_small_body<1, 2, LB>(A, dy, V, partial, split, kt, dys, vs); break;
        default: wgrad_small_body<1, 1, LB>(A, dy, V, partial, split, kt, dys, vs); break;
    }
}

// sum of the partial dU over the splits, in split order
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ partial, float* __restrict__ sum,
                                                           long long n, int splits)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    // eight running sums so that eight loads are in flight; the order of the additions is fixed
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int s = 0;
    for (; s + 8 <= splits; s += 8) {
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] += partial[(size_t)(s + u) * n + e];
    }
    for (; s < splits; ++s) v[0] += partial[(size_t)s * n + e];
    sum[e] = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
}

// ---- step 4: dw = G^T (sum of partial dU) G, one thread per (row of a class, filter) ----
__device__ __forceinline__ float gt_col(int l, int a, const float u[4])
{
    if (l == 3) return a == 0 ? u[0] + 0.5f * (u[1] + u[2]) : a == 1 ? 0.5f * (u[1] - u[2]) : 0.5f * (u[1] + u[2]) + u[3];
    if (l == 2) return a == 0 ? u[0] + u[1] : u[1] + u[2];
    return u[0] + u[1];
}

__global__ __launch_bounds__(256) void wgrad_final_kernel(DevPlan P, WgradArgs A, const float* __restrict__ partial,
                                                          float* __restrict__ dw)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    const int k = blockIdx.y;
    if (row >= P.rows_total) return;
    int qi = 0;
    while (qi + 1 < P.ncls && row >= P.cls[qi + 1].row0) ++qi;
    const DevClass q = P.cls[qi];
    const int l = row - q.row0;
    if (l >= q.L) return;
    const int slot = l / P.C, c = l - slot * P.C;
    const int ai = slot / q.wn, bi = slot - ai * q.wn;
    const DevPiece hp = P.ph[q.h0 + ai], wp = P.pw[q.w0 + bi];
    const int tw = q.lw + 1;
    float u[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float v = 0.f;
            if (i <= q.lh && j <= q.lw) {
                const int p = q.plane0 + i * tw + j;
                const float* src = partial + (size_t)A.poff64[p] * 64 + (size_t)k * A.lstride[p] + l;
                // four loads in flight at a time; the additions keep their order
                int s = 0;
                for (; s + 4 <= A.splits; s += 4) {
                    const float a0 = src[(size_t)s * A.split_floats], a1 = src[(size_t)(s + 1) * A.split_floats];
                    const float a2 = src[(size_t)(s + 2) * A.split_floats], a3 = src[(size_t)(s + 3) * A.split_floats];
                    v = (((v + a0) + a1) + a2) + a3;
                }
                for (; s < A.splits; ++s) v += src[(size_t)s * A.split_floats];
            }
            u[i][j] = v;
        }
    // columns (G_h^T u), then rows ((.) G_w)
    float t[3][4];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float col[4] = {u[0][j], u[1][j], u[2][j], u[3][j]};
            t[a][j] = a < q.lh ? gt_col(q.lh, a, col) : 0.f;
        }
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b)
            if (a < hp.lr && b < wp.lr) {  // (a widened piece's third tap is not its own)
                const int r = P.s * (hp.j + a) + hp.p, s2 = P.s * (wp.j + b) + wp.p;
                dw[(((size_t)k * P.C + c) * P.R + r) * P.S + s2] = gt_col(q.lw, b, t[a]);
            }
}

// The same with whole records: a workgroup owns one filter and 64 channels, its waves walk the parts
// (a wave = one part x 64 channels, loads coalesced along c), the taps go to an LDS copy of the 64
// records dw[k][c0..c0+63][R][S], which are contiguous in memory and written out coalesced -- the
// kernel above writes every record in 4-byte pieces from workgroups far apart in time.
__global__ __launch_bounds__(256) void wgrad_final_lds_kernel(DevPlan P, WgradArgs A, const float* __restrict__ partial,
                                                              float* __restrict__ dw)
{
    extern __shared__ float rec[];  // [64][R * S]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c0 = blockIdx.x * 64, k = blockIdx.y;
    const int c = c0 + lane, RS = P.R * P.S;
    int part0 = 0;
    for (int qi = 0; qi < P.ncls; ++qi) {
        const DevClass q = P.cls[qi];
        const int tw = q.lw + 1, nslot = q.hn * q.wn;
        for (int slot = 0; slot < nslot; ++slot) {
            if (((part0 + slot) & 3) != wave) continue;
            const int ai = slot / q.wn, bi = slot - ai * q.wn;
            const DevPiece hp = P.ph[q.h0 + ai], wp = P.pw[q.w0 + bi];
            const int l = slot * P.C + min(c, P.C - 1);
            float u[4][4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float v = 0.f;
                    if (i <= q.lh && j <= q.lw) {
                        const int p = q.plane0 + i * tw + j;
                        const float* src = partial + (size_t)A.poff64[p] * 64 + (size_t)k * A.lstride[p] + l;
                        int s = 0;
                        for (; s + 4 <= A.splits; s += 4) {
                            const float a0 = src[(size_t)s * A.split_floats], a1 = src[(size_t)(s + 1) * A.split_floats];
                            const float a2 = src[(size_t)(s + 2) * A.split_floats], a3 = src[(size_t)(s + 3) * A.split_floats];
                            v = (((v + a0) + a1) + a2) + a3;
                        }
                        for (; s < A.splits; ++s) v += src[(size_t)s * A.split_floats];
                    }
                    u[i][j] = v;
                }
            float t[3][4];
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float col[4] = {u[0][j], u[1][j], u[2][j], u[3][j]};
                    t[a][j] = a < q.lh ? gt_col(q.lh, a, col) : 0.f;
                }
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b)
                    if (a < hp.lr && b < wp.lr) {  // (a widened piece's third tap is not its own)
                        const int r = P.s * (hp.j + a) + hp.p, s2 = P.s * (wp.j + b) + wp.p;
                        rec[lane * RS + r * P.S + s2] = gt_col(q.lw, b, t[a]);
                    }
        }
        part0 += nslot;
    }
    __syncthreads();
    const int n = min(64, P.C - c0) * RS;
    float* out = dw + ((size_t)k * P.C + c0) * RS;
    for (int i = threadIdx.x; i < n; i += 256) out[i] = rec[i];
}

}  // namespace dwm

struct dwm_bwd_filter_plan {
    dwm_plan_t* fwd;
    double direct_flops, winograd_flops;  // of the layer as the paper splits it
    dwm::WgradArgs a;
    size_t fwd_ws_bytes, dm_bytes, partial_bytes;
    float* ws;
    // short-reduction form (every class has at most 32 rows): one launch for all classes of 16 rows, one for those of 32
    bool small;
    int small_kt;                      // 64-filter tiles
    size_t sum_bytes;                  // the summed dU after the partials
    int n_pass;                        // passes: (class, rows r0 .. r0 + 16 * lb) with lb in {1, 2}
    int pass_lb[2 * dwm::kMaxClasses], pass_code[2 * dwm::kMaxClasses];
    dwm::SmallArgs sc[2 * dwm::kMaxClasses];
};

namespace dwm {

// One launch for the classes whose planes have 16 * lb rows.
static dwm_status_t launch_small_all(int lb, const SmallAllArgs& aa, hipStream_t s, const float* dy, const float* V,
                                     float* partial)
{
    int planes = 0;  // the largest class decides the LDS for V: two chunks of planes * lb * 16 rows x 16 tiles
    for (int i = 0; i < aa.ncls; ++i) planes = std::max(planes, (aa.code[i] / 4 + 1) * (aa.code[i] % 4 + 1));
    const int lds = 2 * planes * lb * 16 * 16 * (int)sizeof(float);
    const dim3 grid((unsigned)((aa.splits + 7) / 8 * 8 * aa.nkt * aa.ncls));
    if (lb == 2) {
        auto kernel = wgrad_small_all_kernel<2>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
        if (attr != hipSuccess) return DWM_ERR_HIP;
        hipLaunchKernelGGL(kernel, grid, dim3(256), lds, s, aa, dy, V, partial);
    } else {
        hipLaunchKernelGGL(wgrad_small_all_kernel<1>, grid, dim3(256), lds, s, aa, dy, V, partial);
    }
    return DWM_OK;
}

// The short-reduction form applies when every class has at most max_rows (padded) rows -- 32, or 64 in two
// passes for the plan that puts all parts in one class -- and there are enough tiles to fill the chip (on a
// small layer the GEMM form's four launches are faster).  The tiles are cut into ranges so that the
// workgroups of ONE class would put two workgroups on every CU; all passes of one row-block count go out
// in one launch, several rounds deep.
static bool small_setup(dwm_bwd_filter_plan& bp, int max_rows)
{
    const DevPlan& d = bp.fwd->d;
    if (d.T < 16384) return false;
    int n1 = 0, n2 = 0;  // passes of one / two row blocks
    for (int c = 0; c < d.ncls; ++c) {
        const int blocks = d.cls[c].Lpad / 16;
        if (blocks * 16 > max_rows) return false;
        n2 += blocks / 2;
        n1 += blocks & 1;
    }
    if (n1 > kMaxClasses || n2 > kMaxClasses) return false;
    WgradArgs& a = bp.a;
    const long long t16 = ((long long)d.T + 15) / 16 * 16;
    const int small_kt = a.Kp / 64;
    long long want = std::max(1, 2 * kNumCUs / small_kt);
    long long per = (t16 + want - 1) / want;
    per = std::max<long long>(64, (per + 15) / 16 * 16);
    const long long nsplit = (t16 + per - 1) / per;
    if (per > 0x7fffffffLL || nsplit > 65535 * 16) return false;
    // (the plan's state is touched only once nothing can fail any more: if this form is refused, the GEMM form
    // must find its own offsets untouched)
    long long total = 0;
    for (int c = 0; c < d.ncls; ++c) total += (long long)(d.cls[c].lh + 1) * (d.cls[c].lw + 1) * a.Kp * d.cls[c].Lpad;
    if (total * nsplit > (1LL << 40)) return false;
    long long off = 0;
    bp.small_kt = small_kt;
    bp.n_pass = 0;
    for (int c = 0; c < d.ncls; ++c) {
        const DevClass& q = d.cls[c];
        const int planes = (q.lh + 1) * (q.lw + 1);
        for (int r0 = 0; r0 < q.Lpad; r0 += 32) {  // rows r0 .. r0+31, or the last 16
            SmallArgs& sa = bp.sc[bp.n_pass];
            sa = SmallArgs{};
            sa.K = d.K; sa.Kp = a.Kp; sa.T = d.T; sa.OH = d.OH; sa.OW = d.OW; sa.TH = d.TH; sa.TW = d.TW;
            sa.vblock_rows = d.vblock_rows; sa.vrow0 = q.v_row0; sa.Lpad = q.Lpad; sa.L = q.L; sa.r0 = r0;
            sa.tiles_per_split = (int)per;
            sa.poff = (int)off;
            sa.div_tiles.init((unsigned)(d.TH * d.TW));
            sa.div_tw.init((unsigned)d.TW);
            bp.pass_lb[bp.n_pass] = q.Lpad - r0 >= 32 ? 2 : 1;
            bp.pass_code[bp.n_pass] = q.lh * 4 + q.lw;
            ++bp.n_pass;
        }
        for (int pl = 0; pl < planes; ++pl) {
            a.poff64[q.plane0 + pl] = (int)((off + (long long)pl * a.Kp * q.Lpad) / 64);
            a.lstride[q.plane0 + pl] = q.Lpad;
        }
        off += (long long)planes * a.Kp * q.Lpad;
    }
    for (int c = 0; c < bp.n_pass; ++c) bp.sc[c].split_floats = off;
    a.split_floats = off;
    a.splits = (int)nsplit;  // what the plan reports; the final kernel reads the summed dU (one "split")
    bp.dm_bytes = 0;
    bp.partial_bytes = ((size_t)nsplit * off * sizeof(float) + 255) / 256 * 256;
    bp.sum_bytes = ((size_t)off * sizeof(float) + 255) / 256 * 256;
    bp.fwd->skip_pad_rows = true;  // the class kernels supply the zero rows themselves
    return true;
}

}  // namespace dwm

namespace dwm {
// dw = G^T (sum of partial dU) G: whole records through LDS where 64 of them fit and the layer has them
static void launch_final(const DevPlan& d, const WgradArgs& a, const float* partial, float* dw, hipStream_t s)
{
    const size_t lds = (size_t)64 * d.R * d.S * sizeof(float);
    if (lds <= 48 * 1024 && d.C >= 32) {  // (with few channels most of the 64 lanes would idle)
        hipLaunchKernelGGL(wgrad_final_lds_kernel, dim3((d.C + 63) / 64, d.K), dim3(256), lds, s, d, a, partial, dw);
    } else {
        hipLaunchKernelGGL(wgrad_final_kernel, dim3((d.rows_total + 255) / 256, d.K), dim3(256), 0, s, d, a, partial, dw);
    }
}
}  // namespace dwm

extern "C" {

// Everything the filter gradient derives from a forward plan (which it takes over, also on failure).
static dwm_status_t wgrad_build(dwm_bwd_filter_plan_t** out, dwm_plan_t* fwd, int K, int small_max_rows)
{
    using namespace dwm;
    dwm_bwd_filter_plan* bp = new (std::nothrow) dwm_bwd_filter_plan;
    if (!bp) {
        dwm_plan_destroy(fwd);
        return DWM_ERR_ALLOC;
    }
    bp->fwd = fwd;
    bp->ws = nullptr;
    bp->direct_flops = fwd->info.direct_flops;
    bp->winograd_flops = fwd->info.winograd_flops;
    WgradArgs& a = bp->a;
    a = WgradArgs{};
    const DevPlan& d = fwd->d;
    a.K = K; a.Kp = (K + 63) / 64 * 64; a.T = d.T; a.tblocks = (d.T + 63) / 64;
    a.n_planes = fwd->planes.n;
    a.dm_rows = a.n_planes * a.Kp;
    a.vblock_rows = d.vblock_rows;
    long long tiles = 0, floats64 = 0;
    for (int p = 0; p < a.n_planes; ++p) {
        const DevPlaneEntry& e = fwd->planes.e[p];
        a.nlt[p] = (e.Lpad + 63) / 64;
        a.lstride[p] = a.nlt[p] * 64;
        a.vrow[p] = (int)e.v_off64;
        a.tile0[p] = (int)tiles;
        a.poff64[p] = (int)floats64;
        tiles += (long long)(a.Kp / 64) * a.nlt[p];
        floats64 += (long long)a.Kp * a.nlt[p];
    }
    a.tile0[a.n_planes] = (int)tiles;
    a.n_tiles = (int)tiles;
    a.split_floats = floats64 * 64;
    // How many ranges the tile axis is cut into.  The chip holds 2 workgroups per CU at a time, so
    // the launch runs in ceil(tiles*splits / 512) rounds of ceil(tblocks/splits) chunks each
    // (2.1 us per chunk-round measured: two workgroups share a CU's matrix cores), and every range
    // writes a partial dU that is read back once (priced at 4 TB/s).  Never fewer than four blocks
    // of tiles per range.
    long long splits = 1;
    {
        const long long max_splits = std::max(1LL, std::min<long long>(32, (a.tblocks + 3) / 4));
        const double partial_us = 2.0 * (double)floats64 * 64 * sizeof(float) / 4e6;
        double best = 0.0;
        for (long long sp = 1; sp <= max_splits; ++sp) {
            const long long rounds = (tiles * sp + 2 * kNumCUs - 1) / (2 * kNumCUs);
            const long long chunks = (a.tblocks + sp - 1) / sp;
            const double t = 2.1 * (double)(rounds * chunks) + partial_us * (double)sp;
            if (sp == 1 || t < best * 0.97) {  // a further cut must pay for itself clearly
                best = t;
                splits = sp;
            }
        }
    }
    a.chunks_per_split = (int)((a.tblocks + splits - 1) / splits);
    a.splits = (a.tblocks + a.chunks_per_split - 1) / a.chunks_per_split;
    const long long lim = (1LL << 31) - 1;
    if (tiles * a.splits > lim || a.split_floats > lim * 16 || (long long)a.tblocks * a.dm_rows > lim) {
        dwm_plan_destroy(fwd);
        delete bp;
        return DWM_ERR_UNSUPPORTED;
    }
    // V, then 64 rows of slack (the last plane's 64-row tile may overhang its rows), dM, partial dU
    bp->fwd_ws_bytes = (dwm_plan_workspace_bytes(fwd) + (size_t)64 * 64 * sizeof(float) + 255) / 256 * 256;
    bp->dm_bytes = ((size_t)a.tblocks * a.dm_rows * 64 * sizeof(float) + 255) / 256 * 256;
    bp->partial_bytes = (size_t)a.splits * a.split_floats * sizeof(float);
    bp->sum_bytes = 0;
    bp->small = small_setup(*bp, small_max_rows);
    *out = bp;
    return DWM_OK;
}

// MFMAs per 16 tiles and 16 filters of the short-reduction form: planes x row blocks, summed over classes
static int small_cost(const dwm_bwd_filter_plan& bp)
{
    const dwm::DevPlan& d = bp.fwd->d;
    int c = 0;
    for (int i = 0; i < d.ncls; ++i) c += (d.cls[i].lh + 1) * (d.cls[i].lw + 1) * (d.cls[i].Lpad / 16);
    return c;
}

dwm_status_t dwm_bwd_filter_plan_destroy(dwm_bwd_filter_plan_t* plan);

dwm_status_t dwm_bwd_filter_plan_create(dwm_bwd_filter_plan_t** out, int N, int C, int H, int W, int K, int R, int S,
                                        int stride, int pad)
{
    using namespace dwm;
    if (!out) return DWM_ERR_INVALID_ARG;
    dwm_plan_t* fwd = nullptr;
    dwm_status_t st = dwm_plan_create(&fwd, N, C, H, W, K, R, S, stride, pad);
    if (st != DWM_OK) return st;
    dwm_bwd_filter_plan* bp = nullptr;
    st = wgrad_build(&bp, fwd, K, 32);
    if (st != DWM_OK) return st;
    if (bp->small) {
        // Short-reduction form: would all parts on the 16 planes of F(2,3)^2 -- two-tap pieces transformed
        // as three-tap ones -- take fewer MFMAs?  Then dy is also read by one class instead of several.
        PlanSpec sp{};
        sp.N = N; sp.C = C; sp.H = H; sp.W = W; sp.K = K; sp.R = R; sp.S = S; sp.stride = stride;
        sp.pad_h = sp.pad_w = pad;
        sp.OH = bp->fwd->d.OH; sp.OW = bp->fwd->d.OW;
        sp.om = bp->fwd->d.om;
        dwm_plan_t* wide = nullptr;
        dwm_bwd_filter_plan* bw = nullptr;
        if (plan_from_spec_widened(&wide, sp) == DWM_OK && wgrad_build(&bw, wide, K, 64) == DWM_OK) {
            if (bw->small && small_cost(*bw) < small_cost(*bp)) {
                bw->direct_flops = bp->direct_flops;
                bw->winograd_flops = bp->winograd_flops;
                std::swap(bp, bw);
            }
            dwm_bwd_filter_plan_destroy(bw);
        }
    }
    *out = bp;
    return DWM_OK;
}

dwm_status_t dwm_bwd_filter_plan_destroy(dwm_bwd_filter_plan_t* plan)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    dwm_plan_destroy(plan->fwd);
    delete plan;
    return DWM_OK;
}

dwm_status_t dwm_bwd_filter_plan_info(const dwm_bwd_filter_plan_t* plan, dwm_bwd_filter_info_t* info)
{
    if (!plan || !info) return DWM_ERR_INVALID_ARG;
    info->n_planes = plan->a.n_planes;
    info->n_tiles = plan->a.n_tiles;
    info->splits = plan->a.splits;
    info->direct_flops = plan->direct_flops;
    info->winograd_flops = plan->winograd_flops;
    return DWM_OK;
}

size_t dwm_bwd_filter_workspace_bytes(const dwm_bwd_filter_plan_t* plan)
{
    return plan ? plan->fwd_ws_bytes + plan->dm_bytes + plan->partial_bytes + plan->sum_bytes : 0;
}

dwm_status_t dwm_bwd_filter_set_workspace(dwm_bwd_filter_plan_t* plan, void* ws_dev, size_t bytes)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    if (!ws_dev || ((uintptr_t)ws_dev & 255u) || bytes < dwm_bwd_filter_workspace_bytes(plan)) return DWM_ERR_WORKSPACE;
    const dwm_status_t st = dwm_plan_set_workspace(plan->fwd, ws_dev, plan->fwd_ws_bytes);
    if (st != DWM_OK) return st;
    plan->ws = static_cast<float*>(ws_dev);
    return DWM_OK;
}

dwm_status_t dwm_conv_backward_filter(const dwm_bwd_filter_plan_t* plan, const float* x_dev, const float* dy_dev,
                                      float* dw_dev, void* stream)
{
    using namespace dwm;
    if (!plan || !x_dev || !dy_dev || !dw_dev) return DWM_ERR_INVALID_ARG;
    if (!plan->ws) return DWM_ERR_WORKSPACE;
    const WgradArgs& a = plan->a;
    const DevPlan& d = plan->fwd->d;
    hipStream_t s = (hipStream_t)stream;
    float* V = plan->ws;
    float* dM = plan->ws + plan->fwd_ws_bytes / sizeof(float);
    float* partial = dM + plan->dm_bytes / sizeof(float);
    // 1. V = B^T d B (and zeros in the columns past the last tile)
    dwm_status_t st = dwm_input_transform(plan->fwd, x_dev, stream);
    if (st != DWM_OK) return st;
    if (d.T & 63) {
        hipLaunchKernelGGL(wgrad_zero_tail_kernel, dim3(64), dim3(256), 0, s,
                           V + (size_t)(a.tblocks - 1) * a.vblock_rows * 64, a.vblock_rows, d.T & 63);
    }
    if (plan->small) {
        // 2'. per class: partial dU straight from dy and V; 3'. their sum; 4. dw = G^T (sum) G
        float* sum = partial + plan->partial_bytes / sizeof(float);
        for (int lb = 1; lb <= 2; ++lb) {
            SmallAllArgs aa{};
            aa.nkt = plan->small_kt;
            aa.splits = a.splits;
            for (int c = 0; c < plan->n_pass; ++c)
                if (plan->pass_lb[c] == lb) {
                    aa.code[aa.ncls] = plan->pass_code[c];
                    aa.c[aa.ncls++] = plan->sc[c];
                }
            if (aa.ncls > 0 && launch_small_all(lb, aa, s, dy_dev, V, partial) != DWM_OK) return DWM_ERR_HIP;
        }
        hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((a.split_floats + 255) / 256)), dim3(256), 0, s, partial,
                           sum, a.split_floats, a.splits);
        WgradArgs fa = a;
        fa.splits = 1;
        launch_final(d, fa, sum, dw_dev, s);
        return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
    }
    // 2. dM = A dY A^T
    const DyShape ds{d.T, d.K, a.Kp, d.TH, d.TW, d.OH, d.OW, a.dm_rows};
    if (d.OW % 4 == 0 && (reinterpret_cast<uintptr_t>(dy_dev) & 15) == 0) {
        hipLaunchKernelGGL(wgrad_dy_transform2_kernel, dim3(a.tblocks, a.Kp / 8), dim3(256), 0, s, ds, plan->fwd->planes,
                           dy_dev, dM);
    } else {
        hipLaunchKernelGGL(wgrad_dy_transform_kernel, dim3(a.tblocks, a.Kp / 4), dim3(256), 0, s, ds, plan->fwd->planes,
                           dy_dev, dM);
    }
    // 3. partial dU
    constexpr int NS = 2;
    constexpr int lds_bytes = NS * 2 * 64 * 64 * 4;
    auto kernel = wgrad_gemm_kernel<NS>;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (attr != hipSuccess) return DWM_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.n_tiles * a.splits)), dim3(256), lds_bytes, s, a, dM, V, partial);
    // 4. dw = G^T (sum) G
    launch_final(d, a, partial, dw_dev, s);
    return hipGetLastError() == hipSuccess ? DWM_OK : DWM_ERR_HIP;
}

}  // extern "C"
