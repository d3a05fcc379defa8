// Host planner and C ABI of libdwm: the "Splitting" step on the kernel side
// (paper Sec. 4.1: eq. 12 groups taps by index modulo the stride, eq. 8 cuts each group
// into consecutive runs of three) plus the bookkeeping that lays the Winograd-domain
// planes out in memory.  Pure integer logic; no GPU call is made in this file.
#include <cstdlib>
#include <cstring>
#include <new>

#include "plan.hpp"

namespace {

using namespace dwm;

long long round_up(long long v, long long a) { return (v + a - 1) / a * a; }

// Split one kernel dimension of r taps at stride s into pieces, longest class first.
// Within a phase the taps are cut 3,3,...,remainder from the low end (eq. 8; the number
// of cuts is ceil(n/3)).  Returns the piece count or -1 if it exceeds kMaxPieces.
// `even_tail`: a remainder of one tap is avoided where the phase has more than one tap --
// 3+1 becomes 2+2, which costs the same number of multiplications (4+2 = 3+3) -- so that
// one-tap pieces, which cannot share frequencies with the others, only arise from phases
// that hold a single tap.
int split_dimension(int r, int s, bool even_tail, bool widen2, DevPiece* out, int start[4], int count[4])
{
    DevPiece tmp[kMaxPieces];
    int n = 0;
    const int phases = s < r ? s : r;  // phases beyond the kernel length hold no tap
    for (int p = 0; p < phases; ++p) {
        const int taps = (r - p + s - 1) / s;
        for (int j = 0; j < taps;) {
            if (n == kMaxPieces) return -1;
            const int rest = taps - j;
            int len = rest < 3 ? rest : 3;
            if (even_tail && rest == 4) len = 2;
            tmp[n++] = DevPiece{p, j, (widen2 && len == 2) ? 3 : len, len};
            j += len;
        }
    }
    int m = 0;
    for (int len = 3; len >= 1; --len) {
        start[len] = m;
        for (int i = 0; i < n; ++i)
            if (tmp[i].l == len) out[m++] = tmp[i];
        count[len] = m - start[len];
    }
    return n;
}

// A^T of F(2,l), row a, column f (Sec. 3.2 for l=3; the 2-tap and 1-tap cases use the
// three- and two-multiplication forms whose entries are all 0/1).
int at_entry(int l, int a, int f)
{
    static const int AT3[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};
    static const int AT2[2][3] = {{1, 1, 0}, {0, 1, 1}};
    static const int AT1[2][2] = {{1, 0}, {0, 1}};
    return l == 3 ? AT3[a][f] : l == 2 ? AT2[a][f] : AT1[a][f];
}

// 64x64 tiles; the deepest reduction chunk the padding allows, except that long launches take 32-step chunks in three
// stages: 48 KB of LDS instead of 64, so a CU holds three workgroups, and a chunk's loads have a whole chunk to land
// in.  "Long" is three or more rounds of whole tiles (a tile's start-up and stores hide behind two others: measured
// 3-10 % faster on 784- and 1568-tile layers) or, above one tile per CU, a reduction of 8192 rows or more per tile
// (rows = all planes' padded reductions; measured with 392 tiles: 25 600 rows 0.806 -> 0.765 ms, 3200 rows 0.130 ->
// 0.132 ms; with at most one tile per CU every tile is cut into ranges of its own and the deep chunks measure 1-7 %
// faster on 100- to 256-tile layers).
int default_contract_variant(int lgran, long long K, long long T, long long rows)
{
    const long long tiles = ((K + 63) / 64) * ((T + 63) / 64);
    return lgran >= 64 ? (tiles >= 3 * dwm::kNumCUs || (tiles > dwm::kNumCUs && rows >= 8192) ? 11 : 12) : lgran >= 32 ? 11 : 10;
}

long long plane_rows(const dwm_plan& p)
{
    long long rows = 0;
    for (int i = 0; i < p.planes.n; ++i) rows += p.planes.e[i].Lpad;
    return rows;
}

}  // namespace

namespace dwm {

bool contract_geometry(const dwm_plan& p, int variant, ContractGeometry* out)
{
    const ContractVariant* cv = nullptr;
    for (int i = 0; i < kNumContractVariants; ++i)
        if (kContractVariants[i].id == variant) cv = &kContractVariants[i];
    if (!cv || p.lgran % cv->lc != 0) return false;
    ContractGeometry g{};
    g.variant = variant;
    g.nkt = (p.d.K + cv->kt() - 1) / cv->kt();
    g.ntt = (p.d.T + cv->tt() - 1) / cv->tt();
    const long long ntiles = (long long)g.nkt * g.ntt;
    if (ntiles > 0x3fffffffLL) return false;
    g.ntiles = (int)ntiles;
    g.full8 = 8 * g.nkt * (g.ntt / 8);
    long long n_iter = 0;
    for (int i = 0; i < p.planes.n; ++i) n_iter += p.planes.e[i].Lpad / cv->lc;
    if (n_iter > 0x3fffffLL) return false;
    g.n_iter = (int)n_iter;
    // Whole tiles for as many full rounds of the CUs as there are; the rest (less than one
    // tile per CU) is cut into equal iteration ranges unless it nearly fills a round anyway.
    g.n_full = g.ntiles / kNumCUs * kNumCUs;
    int rest = g.ntiles - g.n_full;
    if (rest * 10 >= kNumCUs * 9 || p.sk_mode == 2) { g.n_full = g.ntiles; rest = 0; }
    long long sk_slots = kNumCUs;
    if (p.sk_mode == 1 && rest > 0 && g.n_full == kNumCUs) {
        // one full round plus a remainder: two EQUAL ranges per CU instead of a whole tile and
        // a shorter range, so that the two resident workgroups of a CU finish together
        g.n_full = 0;
        rest = g.ntiles;
        sk_slots = 2 * kNumCUs;
    }
    // Fewer tiles than CUs but at least half as many: whole tiles as well.  Splitting EVERY tile
    // (there is no full round whose workgroups share the CUs with the ranges) costs more in
    // partial outputs and their summing than the idle CUs do: measured 0.42 -> 0.26 ms on the
    // four sub-convolutions of the stride-2 layer's data gradient.
    if (g.n_full == 0 && rest * 2 >= kNumCUs && sk_slots == kNumCUs) { g.n_full = g.ntiles; rest = 0; }
    // At most one tile per CU, and long tiles: as whole tiles (or as one flattened range per CU) a
    // CU's four SIMDs would run one wave each, with nothing to issue while that wave waits at a
    // barrier or for LDS.  Every tile is cut into 2..8 ranges of its own instead -- two workgroups
    // per CU, in as few and as full rounds as possible, no range shorter than 16 chunks (measured on
    // 256-tile layers: 58 % -> 77-86 % of the MFMA peak; on a 128-tile layer: 30 % -> 78 %); ranges that do not
    // straddle tiles keep the K tiles of a T tile in step on one XCD, sharing V in its L2.
    // (single precision only: the half-precision contraction is bound by operand delivery, not by
    // issue gaps, and lost 8-60 % with its tiles cut this way)
    g.sk_f = 0;
    if (p.sk_mode == 0 && variant < kFirstHalfVariant && g.ntiles <= kNumCUs && g.n_iter >= 32) {
        // the cut that needs the least time: rounds of two workgroups per CU, each round one range long
        // (plus a little per range for its partial output)
        int f = 1;
        double best = 1e30;
        for (int c = 2; c <= 8 && c <= g.n_iter / 16; ++c) {
            const int rounds = (g.ntiles * c + 2 * kNumCUs - 1) / (2 * kNumCUs);
            const double t = (double)rounds / c + 0.004 * c;
            if (t < best) { best = t; f = c; }
        }
        if (f >= 2) {
            g.sk_f = f;
            g.n_full = 0;
            rest = g.ntiles;
        }
    }
    g.n_sk_tiles = rest;
    if (g.sk_f > 0) {
        g.sk_ipw = (g.n_iter + g.sk_f - 1) / g.sk_f;
        g.sk_wgs = rest * g.sk_f;
        g.sk_maxc = g.sk_f;
        g.partial_floats = (size_t)rest * g.sk_maxc * cv->kt() * cv->tt() * 4;
    } else if (rest > 0) {
        const long long total = (long long)rest * g.n_iter;
        long long wgs = total < sk_slots ? total : sk_slots;
        long long ipw = (total + wgs - 1) / wgs;
        // a tile is shared by at most about four workgroups: beyond that the summing of
        // partial outputs costs more than the balance gains
        if (ipw * 4 < g.n_iter) ipw = (g.n_iter + 3) / 4;
        wgs = (total + ipw - 1) / ipw;
        g.sk_wgs = (int)wgs;
        g.sk_ipw = (int)ipw;
        g.sk_maxc = (int)((g.n_iter - 1) / ipw) + 2;
        g.partial_floats = (size_t)rest * g.sk_maxc * cv->kt() * cv->tt() * 4;
    }
    *out = g;
    return true;
}

}  // namespace dwm

extern "C" {

// One planning pass with the given splitting policy; *out is set on DWM_OK only.
static dwm_status_t plan_build(dwm_plan_t** out, const dwm::PlanSpec& sp, bool even_tail, bool widen2 = false)
{
    const int N = sp.N, C = sp.C, H = sp.H, W = sp.W, K = sp.K, R = sp.R, S = sp.S, stride = sp.stride;
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || stride < 1 || sp.OH < 1 || sp.OW < 1)
        return DWM_ERR_INVALID_ARG;
    const int lim20 = 1 << 20;
    if (sp.pad_h > lim20 || sp.pad_h < -lim20 || sp.pad_w > lim20 || sp.pad_w < -lim20 || H > lim20 || W > lim20 ||
        sp.OH > lim20 || sp.OW > lim20 || stride > lim20 || R > lim20 || S > lim20)
        return DWM_ERR_UNSUPPORTED;

    dwm_plan* p = new (std::nothrow) dwm_plan;
    if (!p) return DWM_ERR_ALLOC;
    std::memset(p, 0, sizeof(*p));
    DevPlan& d = p->d;
    d.N = N; d.C = C; d.H = H; d.W = W; d.K = K; d.R = R; d.S = S; d.s = stride;
    d.Ph = sp.pad_h; d.Pw = sp.pad_w;
    d.OH = sp.OH; d.OW = sp.OW;
    d.om = sp.om;
    d.TH = (d.OH + 1) / 2;
    d.TW = (d.OW + 1) / 2;
    const long long T = (long long)N * d.TH * d.TW;
    const long long Tpad = round_up(T, kTAlign);
    const long long Kpad = round_up(K, kKAlign);
    const long long lim = (1LL << 31) - 1;

    int sh[4], ch[4], sw[4], cw[4];
    d.nh = split_dimension(R, stride, even_tail, widen2, d.ph, sh, ch);
    d.nw = split_dimension(S, stride, even_tail, widen2, d.pw, sw, cw);
    bool ok = d.nh > 0 && d.nw > 0 && Tpad < lim && (long long)N * K * d.om.YH * d.om.YW < lim && (long long)N * K * d.OH * d.OW < lim &&
              (long long)N * C * H * W < lim && (long long)K * C * R * S < lim;

    // Reduction granularity: the largest of 64/32/16 that costs at most 5 % more padded
    // rows than 16 does (long reductions can then be staged in deeper chunks).
    int lgran = kLAlign;
    if (ok) {
        long long rows[3] = {0, 0, 0};
        const int cand[3] = {64, 32, 16};
        for (int lh = 3; lh >= 1; --lh)
            for (int lw = 3; lw >= 1; --lw) {
                if (!ch[lh] || !cw[lw]) continue;
                const long long L = (long long)ch[lh] * cw[lw] * C;
                for (int g = 0; g < 3; ++g) rows[g] += (lh + 1) * (lw + 1) * round_up(L, cand[g]);
            }
        for (int g = 2; g >= 0; --g)
            if (rows[g] * 100 <= rows[2] * 105) lgran = cand[g];
    }

    long long u_off = 0, v_off = 0, mults = 0;
    int n_parts = 0;
    if (ok) {
        d.T = (int)T; d.Tpad = (int)Tpad; d.Kpad = (int)Kpad;
        for (int lh = 3; lh >= 1; --lh)
            for (int lw = 3; lw >= 1; --lw) {
                if (!ch[lh] || !cw[lw]) continue;
                DevClass& q = d.cls[d.ncls];
                q.lh = lh; q.lw = lw;
                q.h0 = sh[lh]; q.hn = ch[lh]; q.w0 = sw[lw]; q.wn = cw[lw];
                const long long L = (long long)q.hn * q.wn * C;
                const long long Lpad = round_up(L, lgran);
                const int planes = (lh + 1) * (lw + 1);
                // the contraction's DMA addresses a lane's share of a chunk with an unsigned 32-bit
                // byte offset from the chunk's base: up to 128 rows of U (row length Lpad), and one
                // V block (v_off rows of 64 tiles) plus a chunk
                if (Lpad > (1LL << 22)) { ok = false; break; }
                q.L = (int)L; q.Lpad = (int)Lpad;
                q.row0 = d.rows_total; q.plane0 = p->planes.n;
                q.u_off = u_off; q.v_row0 = (int)v_off;
                d.rows_total += q.Lpad;
                for (int fh = 0; fh <= lh; ++fh)
                    for (int fw = 0; fw <= lw; ++fw) {
                        DevPlaneEntry& e = p->planes.e[p->planes.n++];
                        const long long pl = fh * (lw + 1) + fw;
                        e.u_off64 = (uint32_t)((u_off + pl * Kpad * Lpad) / 64);
                        e.v_off64 = (uint32_t)(v_off + pl * Lpad);
                        e.Lpad = q.Lpad;
                        int coef = 0;
                        for (int a = 0; a < 2; ++a)
                            for (int b = 0; b < 2; ++b) {
                                const int v = at_entry(lh, a, fh) * at_entry(lw, b, fw);
                                coef |= (v == 0 ? 0 : v > 0 ? 1 : 3) << (2 * (2 * a + b));
                            }
                        e.coef = coef;
                    }
                u_off += planes * Kpad * Lpad;
                v_off += planes * Lpad;  // rows of a V block so far
                if (u_off >= lim * 32 || v_off * Tpad >= lim * 32 || v_off > (1LL << 23)) { ok = false; break; }
                for (int a = 0; a < q.hn; ++a)
                    for (int b = 0; b < q.wn; ++b) {
                        dwm_part_t& pt = p->parts[n_parts++];
                        pt.phase_h = d.ph[q.h0 + a].p; pt.off_h = d.ph[q.h0 + a].j; pt.len_h = lh;
                        pt.phase_w = d.pw[q.w0 + b].p; pt.off_w = d.pw[q.w0 + b].j; pt.len_w = lw;
                        pt.cls = d.ncls; pt.slot = a * q.wn + b;
                        mults += planes;
                    }
                ++d.ncls;
            }
    }
    if (!ok) {
        delete p;
        return DWM_ERR_UNSUPPORTED;
    }
    p->filter_floats = (size_t)u_off;
    d.vblock_rows = (int)v_off;
    p->v_floats = (size_t)v_off * (size_t)Tpad;
    p->ws = nullptr;
    p->ws_bytes = 0;
    p->lgran = lgran;
    p->variant_input = -1;
    p->variant_forward = -1;
    p->sk_mode = 0;
    p->fused_ok = false;
    if (!dwm::contract_geometry(*p, default_contract_variant(lgran, K, T, plane_rows(*p)), &p->geo)) {
        delete p;
        return DWM_ERR_UNSUPPORTED;
    }

    dwm_plan_info_t& in = p->info;
    in.N = N; in.C = C; in.H = H; in.W = W; in.K = K; in.R = R; in.S = S; in.stride = stride; in.pad = sp.pad_h;
    in.OH = d.OH; in.OW = d.OW; in.TH = d.TH; in.TW = d.TW; in.T = T;
    in.n_parts = n_parts; in.n_classes = d.ncls; in.n_planes = p->planes.n;
    in.mults_per_tile = mults;
    in.direct_flops = 2.0 * N * K * C * R * S * d.OH * d.OW;
    in.winograd_flops = 2.0 * (double)mults * C * K * (double)T;
    in.Kpad = d.Kpad; in.Tpad = d.Tpad;
    in.Vblock = (long long)d.vblock_rows * 64;
    // (the single-kernel path goes with the even-tail splitting only)
    p->fused_ok = even_tail && dwm::fused_setup(*p, &p->fused);
    p->inlds_ok = dwm::input_lds_setup(*p, &p->inlds, 0);
    if (p->fused_ok) {
        // the single-kernel path reads its own copy of the transformed filter (see FusedClass)
        size_t uf = (p->filter_floats + 63) / 64 * 64;
        p->uf_gap = p->filter_floats;
        p->uf_begin = uf;
        for (int i = 0; i < p->fused.nfc; ++i) {
            dwm::FusedClass& fc = p->fused.fc[i];
            fc.uf_off = (long long)uf;
            uf += (size_t)p->fused.nslices * fc.nfh * fc.nfw * fc.rows * 32;
        }
        p->filter_floats = uf;
    }
    *out = p;
    return DWM_OK;
}

}  // extern "C"

namespace dwm {
// The single-kernel path for layers with few input channels wants the splitting without
// one-tap remainders; every other layer is split three taps at a time as eq. 8 writes it.
dwm_status_t plan_from_spec(dwm_plan_t** out, const PlanSpec& sp)
{
    dwm_plan_t* p = nullptr;
    dwm_status_t st = plan_build(&p, sp, true);
    if (st == DWM_OK && !p->fused_ok) {
        delete p;
        p = nullptr;
        st = plan_build(&p, sp, false);
    }
    if (st == DWM_OK) *out = p;
    return st;
}

dwm_status_t plan_from_spec_as_printed(dwm_plan_t** out, const PlanSpec& sp)
{
    return plan_build(out, sp, false);
}

dwm_status_t plan_from_spec_widened(dwm_plan_t** out, const PlanSpec& sp)
{
    return plan_build(out, sp, true, true);
}
}  // namespace dwm

extern "C" {

dwm_status_t dwm_plan_create(dwm_plan_t** out, int N, int C, int H, int W, int K, int R, int S,
                             int stride, int pad)
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
    return dwm::plan_from_spec(out, sp);
}

dwm_status_t dwm_plan_destroy(dwm_plan_t* plan)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    delete plan;
    return DWM_OK;
}

dwm_status_t dwm_plan_info(const dwm_plan_t* plan, dwm_plan_info_t* info)
{
    if (!plan || !info) return DWM_ERR_INVALID_ARG;
    *info = plan->info;
    info->forward_path = plan->use_fused() ? 1 : 0;
    return DWM_OK;
}

dwm_status_t dwm_plan_part(const dwm_plan_t* plan, int i, dwm_part_t* part)
{
    if (!plan || !part || i < 0 || i >= plan->info.n_parts) return DWM_ERR_INVALID_ARG;
    *part = plan->parts[i];
    return DWM_OK;
}

dwm_status_t dwm_plan_class(const dwm_plan_t* plan, int i, dwm_class_t* cls)
{
    if (!plan || !cls || i < 0 || i >= plan->d.ncls) return DWM_ERR_INVALID_ARG;
    const dwm::DevClass& q = plan->d.cls[i];
    cls->len_h = q.lh; cls->len_w = q.lw; cls->n_parts = q.hn * q.wn;
    cls->L = q.L; cls->Lpad = q.Lpad; cls->u_offset = q.u_off; cls->v_offset = (long long)q.v_row0 * 64;
    return DWM_OK;
}

dwm_status_t dwm_plan_fused_info(const dwm_plan_t* plan, int* n_classes, int* n_rows, int* n_slices)
{
    if (!plan || !n_classes || !n_rows || !n_slices) return DWM_ERR_INVALID_ARG;
    *n_classes = plan->fused_ok ? plan->fused.nfc : 0;
    *n_rows = plan->fused_ok ? plan->fused.rows_total : 0;
    *n_slices = plan->fused_ok ? plan->fused.nslices : 0;
    return DWM_OK;
}

dwm_status_t dwm_plan_fused_class(const dwm_plan_t* plan, int i, dwm_fused_class_t* cls)
{
    if (!plan || !cls || !plan->fused_ok || i < 0 || i >= plan->fused.nfc) return DWM_ERR_INVALID_ARG;
    const dwm::FusedClass& fc = plan->fused.fc[i];
    cls->wide_h = fc.wide_h; cls->wide_w = fc.wide_w;
    cls->n_freq_h = fc.nfh; cls->n_freq_w = fc.nfw;
    cls->first_row = fc.row0; cls->rows = fc.rows;
    cls->uf_offset = fc.uf_off;
    return DWM_OK;
}

dwm_status_t dwm_plan_fused_row(const dwm_plan_t* plan, int row, dwm_fused_row_t* out)
{
    if (!plan || !out || !plan->fused_ok || row < 0 || row >= plan->fused.rows_total) return DWM_ERR_INVALID_ARG;
    const unsigned desc = plan->fused.rowdesc[row];
    const dwm::DevPiece hp = plan->d.ph[desc & 15], wp = plan->d.pw[(desc >> 4) & 15];
    out->channel = (int)((desc >> 8) & 127);
    out->real = (int)(desc >> 15);
    out->part = -1;
    for (int i = 0; i < plan->info.n_parts; ++i) {
        const dwm_part_t& pt = plan->parts[i];
        if (pt.phase_h == hp.p && pt.off_h == hp.j && pt.len_h == hp.l && pt.phase_w == wp.p &&
            pt.off_w == wp.j && pt.len_w == wp.l)
            out->part = i;
    }
    return out->part >= 0 ? DWM_OK : DWM_ERR_INVALID_ARG;
}

size_t dwm_plan_filter_bytes(const dwm_plan_t* plan) { return plan ? plan->filter_floats * sizeof(float) : 0; }
size_t dwm_plan_workspace_bytes(const dwm_plan_t* plan) { return plan ? plan->ws_need_bytes() : 0; }

dwm_status_t dwm_plan_set_workspace(dwm_plan_t* plan, void* ws_dev, size_t bytes)
{
    if (!plan) return DWM_ERR_INVALID_ARG;
    if (!ws_dev || ((uintptr_t)ws_dev & 255u) || bytes < plan->ws_need_bytes()) return DWM_ERR_WORKSPACE;
    plan->ws = static_cast<float*>(ws_dev);
    plan->ws_bytes = bytes;
    return DWM_OK;
}

dwm_status_t dwm_plan_set_variant(dwm_plan_t* plan, const char* stage, int variant)
{
    if (!plan || !stage) return DWM_ERR_INVALID_ARG;
    if (!std::strcmp(stage, "input")) {
        if (variant > 3 || (variant >= 2 && !plan->inlds_ok)) return DWM_ERR_INVALID_ARG;
        plan->variant_input = variant;
        return DWM_OK;
    }
    if (!std::strcmp(stage, "input_cg")) {  // channels per workgroup of the LDS-staged input transform
        dwm::InLdsArgs a;
        if (!dwm::input_lds_setup(*plan, &a, variant) || (variant > 0 && a.cg != variant)) return DWM_ERR_INVALID_ARG;
        plan->inlds = a;
        plan->inlds_ok = true;
        return DWM_OK;
    }
    if (!std::strcmp(stage, "forward")) {
        if (variant > 1 || (variant == 1 && !plan->fused_ok)) return DWM_ERR_INVALID_ARG;
        plan->variant_forward = variant;
        return DWM_OK;
    }
    // what follows moves the partial outputs and the arrival counters inside the workspace
    if (plan->ws) return std::strcmp(stage, "split") && std::strcmp(stage, "contract") ? DWM_ERR_INVALID_ARG : DWM_ERR_WORKSPACE;
    if (!std::strcmp(stage, "split")) {  // 0: whole tiles + split remainder, 1: all tiles split evenly
        const int old_mode = plan->sk_mode;
        plan->sk_mode = variant == 1 ? 1 : variant == 2 ? 2 : 0;
        const dwm_status_t st = dwm_plan_set_variant(plan, "contract", plan->geo.variant);
        if (st != DWM_OK) plan->sk_mode = old_mode;
        return st;
    }
    if (std::strcmp(stage, "contract") || variant >= dwm::kFirstHalfVariant) return DWM_ERR_INVALID_ARG;
    dwm::ContractGeometry g;
    if (!dwm::contract_geometry(*plan, variant < 0 ? default_contract_variant(plan->lgran, plan->d.K, plan->d.T, plane_rows(*plan)) : variant, &g))
        return DWM_ERR_INVALID_ARG;
    plan->geo = g;
    return DWM_OK;
}

dwm_status_t dwm_filter_transform(const dwm_plan_t* plan, const float* w_dev, float* Ugw_dev, void* stream)
{
    if (!plan || !w_dev || !Ugw_dev) return DWM_ERR_INVALID_ARG;
    const dwm_status_t st = dwm::launch_filter_transform(*plan, w_dev, Ugw_dev, stream);
    if (st != DWM_OK || !plan->fused_ok) return st;
    return dwm::launch_fused_filter(*plan, w_dev, Ugw_dev, stream);
}

dwm_status_t dwm_input_transform(const dwm_plan_t* plan, const float* x_dev, void* stream)
{
    if (!plan || !x_dev) return DWM_ERR_INVALID_ARG;
    if (!plan->ws) return DWM_ERR_WORKSPACE;
    return dwm::launch_input_transform(*plan, x_dev, plan->ws, stream);
}

dwm_status_t dwm_contract_output(const dwm_plan_t* plan, const float* Ugw_dev, float* y_dev, void* stream)
{
    if (!plan || !Ugw_dev || !y_dev) return DWM_ERR_INVALID_ARG;
    if (!plan->ws) return DWM_ERR_WORKSPACE;
    return dwm::launch_contract_output(*plan, Ugw_dev, plan->ws, y_dev, stream);
}

dwm_status_t dwm_conv_forward(const dwm_plan_t* plan, const float* x_dev, const float* Ugw_dev,
                              float* y_dev, void* stream)
{
    if (!plan || !x_dev || !Ugw_dev || !y_dev) return DWM_ERR_INVALID_ARG;
    if (!plan->ws) return DWM_ERR_WORKSPACE;
    if (plan->use_fused()) return dwm::launch_fused_forward(*plan, x_dev, Ugw_dev, y_dev, stream);
    dwm_status_t st = dwm::launch_input_transform(*plan, x_dev, plan->ws, stream);
    if (st != DWM_OK) return st;
    return dwm::launch_contract_output(*plan, Ugw_dev, plan->ws, y_dev, stream);
}

const char* dwm_status_string(dwm_status_t status)
{
    switch (status) {
        case DWM_OK: return "ok";
        case DWM_ERR_INVALID_ARG: return "invalid argument";
        case DWM_ERR_UNSUPPORTED: return "unsupported shape";
        case DWM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case DWM_ERR_ALLOC: return "host allocation failed";
        case DWM_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
