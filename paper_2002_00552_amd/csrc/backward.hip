// Gradient of the DWM convolution with respect to its input (paper Sec. 3.1 eq. 5 and
// Sec. 4.2 eq. 16-17 state what is computed: every part receives the whole output gradient
// and the parts' input gradients add up -- the sum is the gradient of the ordinary
// convolution).
//
// How it is organised here.  The gradient image is itself a convolution of dy, and the
// stride splitting of Sec. 4.1 (eq. 12-14) applies to it in mirror image: an input pixel at
// padded position u belongs to phase a = u mod stride, only taps r = stride*i + a reach it,
// and with u = stride*u' + a
//     dx_a[u'] = sum_k sum_i dy[k][u' - i] * w[k][c][stride*i + a]
// is a STRIDE-1 convolution of dy with the taps of phase a, flipped, filters and channels
// swapped.  So the gradient is stride^2 independent stride-1 convolutions -- one per phase
// pair (a, b) -- each run through the forward DWM machinery of this library (splitting into
// pieces of at most three taps, F(2,l), the same kernels), whose outputs interleave: the
// sub-convolution of phase (a, b) writes the pixels (stride*o + oy, stride*o' + ox) of dx.
// Every pixel of dx is written exactly once, nothing is accumulated in memory, results are
// bit-identical from run to run.  Phases that hold no tap (stride > kernel) get zeros.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "plan.hpp"

struct dwm_bwd_data_plan {
    int N, C, H, W, K, R, S, s, P, OH, OW;
    struct Phase {
        int a, b, na, nb;    // phase pair, taps per dimension (0: no tap)
        int oy, ox, UH, UW;  // first pixel of the phase in dx, pixels per dimension
        dwm_plan_t* sub;     // stride-1 sub-convolution (null if the phase has no tap or no pixel)
        size_t u_off;        // its transformed filter inside Ugw (floats)
    };
    std::vector<Phase> phases;
    size_t wtmp_floats;      // start of Ugw: scratch for one phase's gathered, flipped weights
    size_t filter_floats, ws_bytes;
    double direct_flops;
    // all sub-convolutions contracted in one launch (contract_batch.hip): each then has its own
    // slice of the workspace, ws_off[i] bytes from its start for phase i
    bool batched;
    int batch_lc;
    dwm::BatchArgs batch;
    dwm::PlaneTable batch_planes;
    std::vector<size_t> ws_off;
    float* ws;
    // ... and, where their tile grids coincide, ONE input transform for all of them: a plan that
    // holds every sub-convolution's pieces and classes (used by the input transform only)
    dwm_plan_t* merged;
    // few input channels: the whole gradient in one kernel (backward_small.hip), its filter copy
    // u_small_off floats into Ugw; variant_path < 0: the planner's choice, 0: sub-convolutions, 1: that kernel
    bool small_ok;
    dwm::BwdSmallArgs small;
    size_t u_small_off;
    int variant_path;
    bool use_small() const { return small_ok && (variant_path == 1 || (variant_path < 0 && small_default)); }
    bool small_default;
};

namespace dwm {

// wt[c][k][i][j] = w[k][c][s*(na-1-i) + a][s*(nb-1-j) + b]
__global__ __launch_bounds__(256) void bwd_gather_weights_kernel(const float* __restrict__ w, float* __restrict__ wt,
                                                                 int K, int C, int R, int S, int s, int a, int b,
                                                                 int na, int nb)
{
    const size_t total = (size_t)C * K * na * nb;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int j = (int)(e % nb);
        const int i = (int)((e / nb) % na);
        const int k = (int)((e / ((size_t)nb * na)) % K);
        const int c = (int)(e / ((size_t)nb * na * K));
        wt[e] = w[(((size_t)k * C + c) * R + (s * (na - 1 - i) + a)) * S + (s * (nb - 1 - j) + b)];
    }
}

// dx[n][c][sy*o + oy][sx*o' + ox] = 0 for o < UH, o' < UW
__global__ __launch_bounds__(256) void bwd_zero_phase_kernel(float* __restrict__ dx, int planes, int H, int W, int s,
                                                             int oy, int ox, int UH, int UW)
{
    const size_t total = (size_t)planes * UH * UW;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int v = (int)(e % UW);
        const int u = (int)((e / UW) % UH);
        const size_t pl = e / ((size_t)UW * UH);
        dx[(pl * H + (size_t)(s * u + oy)) * W + (s * v + ox)] = 0.f;
    }
}

static int ceil_div(int x, int d) { return x >= 0 ? (x + d - 1) / d : -((-x) / d); }

}  // namespace dwm


// (the batch's plane table with every plane pointing into its own sub-convolution's V)
static void setup_batch_unmerged_planes(dwm_bwd_data_plan& bp, const std::vector<int>& subs)
{
    for (int q = 0; q < bp.batch.nprob; ++q) {
        const dwm_plan_t* sp = bp.phases[subs[q]].sub;
        for (int e = 0; e < sp->planes.n; ++e) bp.batch_planes.e[bp.batch.p[q].plane0 + e].v_off64 = sp->planes.e[e].v_off64;
    }
}

// One input transform for all sub-convolutions.  They read the same dy; what differs is which
// window of it a tile of phase (a, b) starts at.  A sub-convolution's patch element is at row
// 2*ty + j + i - Ph_a of dy; with Ph = the largest Ph_a and j' = j + (Ph - Ph_a) that is
// 2*ty + j' + i - Ph for all of them, so one plan can hold the pieces of every phase (those of
// phase a once, shifted), and one class per (sub-convolution, class) whose parts are the products
// of ITS phases' pieces.  The staged rows of dy are then fetched once instead of once per phase.
// Applies when the tile grids coincide and the pieces and classes fit the plan's tables.
static void setup_merged(dwm_bwd_data_plan& bp, const std::vector<int>& subs)
{
    using namespace dwm;
    bp.merged = nullptr;
    const dwm_plan_t* first = bp.phases[subs[0]].sub;
    int Ph = first->d.Ph, Pw = first->d.Pw, ncls = 0;
    for (int i : subs) {
        const DevPlan& d = bp.phases[i].sub->d;
        if (d.TH != first->d.TH || d.TW != first->d.TW || d.T != first->d.T || d.OH != first->d.OH ||
            d.OW != first->d.OW)
            return;
        Ph = std::max(Ph, d.Ph);
        Pw = std::max(Pw, d.Pw);
        ncls += d.ncls;
    }
    if (ncls > kMaxClasses) return;
    dwm_plan* m = new (std::nothrow) dwm_plan;
    if (!m) return;
    std::memset(m, 0, sizeof(*m));
    DevPlan& d = m->d;
    d = first->d;
    d.Ph = Ph; d.Pw = Pw;
    d.nh = d.nw = d.ncls = d.rows_total = d.vblock_rows = 0;
    // pieces: those of phase a (rows) / b (columns) once
    std::vector<int> hoff(bp.s, -1), woff(bp.s, -1);
    bool ok = true;
    for (int i : subs) {
        const auto& ph = bp.phases[i];
        const DevPlan& sd = ph.sub->d;
        if (hoff[ph.a] < 0) {
            if (d.nh + sd.nh > kMaxPieces) { ok = false; break; }
            hoff[ph.a] = d.nh;
            for (int q = 0; q < sd.nh; ++q) {
                DevPiece pc = sd.ph[q];
                pc.j += Ph - sd.Ph;
                d.ph[d.nh++] = pc;
            }
        }
        if (woff[ph.b] < 0) {
            if (d.nw + sd.nw > kMaxPieces) { ok = false; break; }
            woff[ph.b] = d.nw;
            for (int q = 0; q < sd.nw; ++q) {
                DevPiece pc = sd.pw[q];
                pc.j += Pw - sd.Pw;
                d.pw[d.nw++] = pc;
            }
        }
    }
    long long v_off = 0;
    if (ok)
        for (int q = 0; q < bp.batch.nprob && ok; ++q) {
            const auto& ph = bp.phases[subs[q]];
            const DevPlan& sd = ph.sub->d;
            for (int c = 0; c < sd.ncls; ++c) {
                DevClass cl = sd.cls[c];
                const int planes = (cl.lh + 1) * (cl.lw + 1);
                cl.h0 += hoff[ph.a];
                cl.w0 += woff[ph.b];
                cl.row0 = d.rows_total;
                cl.v_row0 = (int)v_off;
                // this class's planes in the batch's table now point into the merged V
                for (int pl = 0; pl < planes; ++pl)
                    bp.batch_planes.e[bp.batch.p[q].plane0 + sd.cls[c].plane0 + pl].v_off64 = (uint32_t)(v_off + (long long)pl * cl.Lpad);
                d.cls[d.ncls++] = cl;
                d.rows_total += cl.Lpad;
                v_off += (long long)planes * cl.Lpad;
                if (v_off * d.Tpad >= ((1LL << 31) - 1) * 32) ok = false;
            }
        }
    if (!ok) {
        delete m;
        setup_batch_unmerged_planes(bp, subs);
        return;
    }
    d.vblock_rows = (int)v_off;
    m->v_floats = (size_t)v_off * (size_t)d.Tpad;
    m->lgran = bp.batch_lc;
    m->variant_input = -1;
    m->variant_forward = 0;
    m->inlds_ok = input_lds_setup(*m, &m->inlds, 0);
    for (int q = 0; q < bp.batch.nprob; ++q) {
        bp.batch.p[q].vblock = d.vblock_rows * 64;
        bp.batch.p[q].v_base = 0;
    }
    bp.ws_bytes = std::max<size_t>((m->v_floats * sizeof(float) + 255) / 256 * 256 + 256, 256);
    bp.merged = m;
}

// One launch for the contractions of all sub-convolutions where that applies: at least two of
// them, all on the staged path, their planes fit one table.  The sub-convolutions are ordered
// longest first; each keeps its own slice of the workspace (its V is alive until the one launch).
static void setup_batch(dwm_bwd_data_plan& bp)
{
    using namespace dwm;
    bp.batched = false;
    bp.merged = nullptr;
    bp.ws = nullptr;
    bp.ws_off.assign(bp.phases.size(), 0);
    std::vector<int> subs;
    int planes = 0, lc = 32;  // 32-step chunks, three stages: 48 KB of LDS, three workgroups per CU (measured best)
    for (size_t i = 0; i < bp.phases.size(); ++i) {
        const dwm_plan_t* sp = bp.phases[i].sub;
        if (!sp) continue;
        if (sp->use_fused()) return;
        subs.push_back((int)i);
        planes += sp->planes.n;
        lc = std::min(lc, sp->lgran);
    }
    if (subs.size() < 2 || subs.size() > (size_t)kMaxBatch || planes > kMaxPlanes) return;
    auto n_iter = [&](int i) {
        int n = 0;
        const PlaneTable& pt = bp.phases[i].sub->planes;
        for (int q = 0; q < pt.n; ++q) n += pt.e[q].Lpad / lc;
        return n;
    };
    std::stable_sort(subs.begin(), subs.end(), [&](int a, int b) { return n_iter(a) > n_iter(b); });
    BatchArgs& A = bp.batch;
    A = BatchArgs{};
    A.K = bp.C;  // the sub-convolutions' filters are the layer's input channels
    A.nkt = (bp.C + 63) / 64;
    A.nprob = (int)subs.size();
    bp.batch_planes = PlaneTable{};
    size_t ws = 0;
    long long tiles = 0;
    for (int q = 0; q < A.nprob; ++q) {
        const int i = subs[q];
        const auto& ph = bp.phases[i];
        const dwm_plan_t* sp = ph.sub;
        if (ph.u_off % 64 != 0) return;
        BatchProb& P = A.p[q];
        P.plane0 = bp.batch_planes.n;
        P.n_iter = n_iter(i);
        P.tile0 = (int)tiles;
        P.vblock = sp->d.vblock_rows * 64;
        P.om = sp->d.om;
        P.OH = sp->d.OH; P.OW = sp->d.OW; P.TH = sp->d.TH; P.TW = sp->d.TW; P.T = sp->d.T;
        P.v_base = (long long)(ws / sizeof(float));
        bp.ws_off[i] = ws;
        ws += (dwm_plan_workspace_bytes(sp) + 255) / 256 * 256;
        for (int e = 0; e < sp->planes.n; ++e) {
            DevPlaneEntry pe = sp->planes.e[e];
            pe.u_off64 += (uint32_t)(ph.u_off / 64);
            bp.batch_planes.e[bp.batch_planes.n++] = pe;
        }
        tiles += (long long)A.nkt * ((sp->d.T + 63) / 64);
    }
    if (tiles > 0x7fffffffLL || ws / sizeof(float) > 0x7fffffffffffLL) return;
    A.ntiles = (int)tiles;
    bp.batch_lc = lc;
    bp.ws_bytes = std::max<size_t>(ws, 256);
    bp.batched = true;
    setup_merged(bp, subs);
}

extern "C" {

dwm_status_t dwm_bwd_data_plan_create(dwm_bwd_data_plan_t** out, int N, int C, int H, int W, int K, int R, int S,
                                      int stride, int pad)
{
    using namespace dwm;
    if (!out) return DWM_ERR_INVALID_ARG;
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return DWM_ERR_INVALID_ARG;
    if ((long long)H + 2LL * pad < R || (long long)W + 2LL * pad < S) return DWM_ERR_INVALID_ARG;
    if (pad > (1 << 20) || H > (1 << 20) || W > (1 << 20) || stride > 8) return DWM_ERR_UNSUPPORTED;
    dwm_bwd_data_plan* bp = new (std::nothrow) dwm_bwd_data_plan;
    if (!bp) return DWM_ERR_ALLOC;
    bp->N = N; bp->C = C; bp->H = H; bp->W = W; bp->K = K; bp->R = R; bp->S = S; bp->s = stride; bp->P = pad;
    bp->OH = (H + 2 * pad - R) / stride + 1;
    bp->OW = (W + 2 * pad - S) / stride + 1;
    bp->direct_flops = 2.0 * N * K * C * R * S * bp->OH * bp->OW;
    bp->wtmp_floats = 0;
    bp->ws_bytes = 256;
    const int s = stride;
    dwm_status_t st = DWM_OK;
    for (int a = 0; a < s && st == DWM_OK; ++a)
        for (int b = 0; b < s && st == DWM_OK; ++b) {
            dwm_bwd_data_plan::Phase ph{};
            ph.a = a; ph.b = b;
            ph.na = a < R ? (R - a + s - 1) / s : 0;
            ph.nb = b < S ? (S - b + s - 1) / s : 0;
            // pixels of this phase: padded position u = s*u' + a with pad <= u < H + pad
            const int u0 = ceil_div(pad - a, s), v0 = ceil_div(pad - b, s);
            const int u1 = H + pad - 1 - a >= 0 ? (H + pad - 1 - a) / s : -1;
            const int v1 = W + pad - 1 - b >= 0 ? (W + pad - 1 - b) / s : -1;
            ph.UH = u1 - u0 + 1; ph.UW = v1 - v0 + 1;
            ph.oy = s * u0 + a - pad; ph.ox = s * v0 + b - pad;
            ph.sub = nullptr;
            if (ph.UH > 0 && ph.UW > 0 && ph.na > 0 && ph.nb > 0) {
                // the stride-1 sub-convolution: dy is its input (K channels), C filters of na x nb
                // taps; output o stands for u' = o + u0, whose window starts at dy row u' - (na-1)
                PlanSpec sp{};
                sp.N = N; sp.C = K; sp.H = bp->OH; sp.W = bp->OW; sp.K = C; sp.R = ph.na; sp.S = ph.nb; sp.stride = 1;
                sp.pad_h = ph.na - 1 - u0; sp.pad_w = ph.nb - 1 - v0;
                sp.OH = ph.UH; sp.OW = ph.UW;
                sp.om = OutMap{H, W, s, ph.oy, s, ph.ox};
                st = plan_from_spec(&ph.sub, sp);
                if (st == DWM_OK) {
                    bp->wtmp_floats = std::max(bp->wtmp_floats, (size_t)C * K * ph.na * ph.nb);
                    bp->ws_bytes = std::max(bp->ws_bytes, dwm_plan_workspace_bytes(ph.sub));
                }
            }
            bp->phases.push_back(ph);
        }
    if (st != DWM_OK) {
        for (auto& ph : bp->phases)
            if (ph.sub) dwm_plan_destroy(ph.sub);
        delete bp;
        return st;
    }
    size_t off = (bp->wtmp_floats + 63) / 64 * 64;
    bp->wtmp_floats = off;
    for (auto& ph : bp->phases)
        if (ph.sub) {
            ph.u_off = off;
            off += (dwm_plan_filter_bytes(ph.sub) / sizeof(float) + 63) / 64 * 64;
        }
    // the single-kernel form: chosen where the sub-convolutions would have only a handful of filters
    bp->small_ok = bwd_small_setup(N, C, H, W, K, R, S, stride, pad, &bp->small);
    // (LDS: room for the workgroups per CU its registers allow -- one where a wave holds several column blocks of
    // sixteen planes, else at least two)
    const size_t small_lds_max = (bp->small.nb > 1 && bp->small.four ? 152 : 78) * 1024;
    bp->small_default = bp->small_ok && C <= 16 && bp->small.nf <= 64 && bp->small.lds_bytes <= small_lds_max &&
                        bp->small.eff_pct >= 50;
    bp->variant_path = -1;
    bp->u_small_off = off;
    if (bp->small_ok) off += (bp->small.u_floats + 63) / 64 * 64;
    bp->filter_floats = off;
    setup_batch(*bp);
    *out = bp;
    return DWM_OK;
}

dwm_status_t dwm_bwd_data_plan_destroy(dwm_bwd_data_plan_t* plan)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    for (auto& ph : plan->phases)
        if (ph.sub) dwm_plan_destroy(ph.sub);
    delete plan->merged;
    delete plan;
    return DWM_OK;
}

dwm_status_t dwm_bwd_data_plan_info(const dwm_bwd_data_plan_t* plan, dwm_bwd_data_info_t* info)
{
    if (!plan || !info) return DWM_ERR_INVALID_ARG;
    info->n_phases = (int)plan->phases.size();
    info->n_subconvs = 0;
    info->winograd_flops = 0.0;
    info->mults_per_input_block = 0;
    for (const auto& ph : plan->phases)
        if (ph.sub) {
            dwm_plan_info_t si;
            dwm_plan_info(ph.sub, &si);
            ++info->n_subconvs;
            info->winograd_flops += si.winograd_flops;
            info->mults_per_input_block += si.mults_per_tile;
        }
    info->direct_flops = plan->direct_flops;
    info->single_kernel = plan->use_small() ? 1 : 0;
    return DWM_OK;
}

dwm_status_t dwm_bwd_data_plan_phase(const dwm_bwd_data_plan_t* plan, int i, dwm_bwd_phase_t* out)
{
    if (!plan || !out || i < 0 || i >= (int)plan->phases.size()) return DWM_ERR_INVALID_ARG;
    const auto& ph = plan->phases[i];
    out->phase_h = ph.a; out->phase_w = ph.b; out->taps_h = ph.na; out->taps_w = ph.nb;
    out->first_h = ph.oy; out->first_w = ph.ox; out->count_h = ph.UH; out->count_w = ph.UW;
    out->has_subconv = ph.sub != nullptr;
    return DWM_OK;
}

dwm_status_t dwm_bwd_data_set_variant(dwm_bwd_data_plan_t* plan, const char* stage, int variant)
{
    if (!plan || !stage) return DWM_ERR_INVALID_ARG;
    if (std::strcmp(stage, "path") != 0) return DWM_ERR_INVALID_ARG;
    if (variant < -1 || variant > 1) return DWM_ERR_INVALID_ARG;
    if (variant == 1 && !plan->small_ok) return DWM_ERR_UNSUPPORTED;
    plan->variant_path = variant;
    return DWM_OK;
}

size_t dwm_bwd_data_filter_bytes(const dwm_bwd_data_plan_t* plan) { return plan ? plan->filter_floats * sizeof(float) : 0; }
size_t dwm_bwd_data_workspace_bytes(const dwm_bwd_data_plan_t* plan) { return plan ? plan->ws_bytes : 0; }

dwm_status_t dwm_bwd_data_set_workspace(dwm_bwd_data_plan_t* plan, void* ws_dev, size_t bytes)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    if (bytes < plan->ws_bytes) return DWM_ERR_WORKSPACE;
    if (plan->merged) {
        if (!ws_dev || ((uintptr_t)ws_dev & 255u)) return DWM_ERR_WORKSPACE;
        plan->merged->ws = static_cast<float*>(ws_dev);
        plan->merged->ws_bytes = bytes;
        plan->ws = static_cast<float*>(ws_dev);
        return DWM_OK;
    }
    for (size_t i = 0; i < plan->phases.size(); ++i) {
        auto& ph = plan->phases[i];
        if (!ph.sub) continue;
        const size_t off = plan->batched ? plan->ws_off[i] : 0;
        const dwm_status_t st = dwm_plan_set_workspace(ph.sub, ws_dev ? static_cast<char*>(ws_dev) + off : nullptr,
                                                       plan->batched ? dwm_plan_workspace_bytes(ph.sub) : bytes);
        if (st != DWM_OK) return st;
    }
    plan->ws = static_cast<float*>(ws_dev);
    return DWM_OK;
}

dwm_status_t dwm_bwd_data_filter_transform(const dwm_bwd_data_plan_t* plan, const float* w_dev, float* Ugw_dev,
                                           void* stream)
{
    // (a layer in which no tap reaches any pixel of dx -- stride above the kernel size on a narrow image -- has no
    // transformed filter at all: zero bytes, and no buffer to ask for)
    if (!plan || !w_dev || (!Ugw_dev && plan->filter_floats > 0)) return DWM_ERR_INVALID_ARG;
    for (const auto& ph : plan->phases) {
        if (!ph.sub) continue;
        const size_t total = (size_t)plan->C * plan->K * ph.na * ph.nb;
        const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
        // the scratch at the start of Ugw is reused phase after phase: stream order keeps it safe
        hipLaunchKernelGGL(dwm::bwd_gather_weights_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, w_dev,
                           Ugw_dev, plan->K, plan->C, plan->R, plan->S, plan->s, ph.a, ph.b, ph.na, ph.nb);
        if (hipGetLastError() != hipSuccess) return DWM_ERR_HIP;
        const dwm_status_t st = dwm_filter_transform(ph.sub, Ugw_dev, Ugw_dev + ph.u_off, stream);
        if (st != DWM_OK) return st;
    }
    if (plan->small_ok)
        return dwm::launch_bwd_small_filter(plan->small, plan->R, plan->S, w_dev, Ugw_dev + plan->u_small_off, stream);
    return DWM_OK;
}

dwm_status_t dwm_conv_backward_data(const dwm_bwd_data_plan_t* plan, const float* dy_dev, const float* Ugw_dev,
                                    float* dx_dev, void* stream)
{
    if (!plan || !dy_dev || (!Ugw_dev && plan->filter_floats > 0) || !dx_dev) return DWM_ERR_INVALID_ARG;
    if (plan->use_small()) return dwm::launch_bwd_small(plan->small, dy_dev, Ugw_dev + plan->u_small_off, dx_dev, stream);
    for (const auto& ph : plan->phases) {
        if (ph.UH <= 0 || ph.UW <= 0) continue;
        if (!ph.sub) {  // no tap reaches these pixels
            const size_t total = (size_t)plan->N * plan->C * ph.UH * ph.UW;
            const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 8192);
            hipLaunchKernelGGL(dwm::bwd_zero_phase_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, dx_dev,
                               plan->N * plan->C, plan->H, plan->W, plan->s, ph.oy, ph.ox, ph.UH, ph.UW);
            if (hipGetLastError() != hipSuccess) return DWM_ERR_HIP;
            continue;
        }
        if (plan->merged) continue;  // one input transform for all of them, below
        if (plan->batched) {  // its input transform now, its contraction with all the others below
            if (!plan->ws) return DWM_ERR_WORKSPACE;
            const dwm_status_t st = dwm::launch_input_transform(*ph.sub, dy_dev, ph.sub->ws, stream);
            if (st != DWM_OK) return st;
            continue;
        }
        const dwm_status_t st = dwm_conv_forward(ph.sub, dy_dev, Ugw_dev + ph.u_off, dx_dev, stream);
        if (st != DWM_OK) return st;
    }
    if (plan->merged) {
        if (!plan->ws) return DWM_ERR_WORKSPACE;
        const dwm_status_t st = dwm::launch_input_transform(*plan->merged, dy_dev, plan->ws, stream);
        if (st != DWM_OK) return st;
    }
    if (plan->batched)
        return dwm::launch_contract_batch(plan->batch, plan->batch_planes, plan->batch_lc, Ugw_dev, plan->ws, dx_dev,
                                          stream);
    return DWM_OK;
}

}  // extern "C"
