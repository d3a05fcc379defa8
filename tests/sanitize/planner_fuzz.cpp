// Host-only fuzz of the planner behind the C ABI, built with -fsanitize=address,undefined by
// tests/test_sanitize.py: plans are created for random and for extreme shapes, every introspection
// call is walked, variants are switched, and the decomposition's invariants are checked.  The
// kernel launchers are stubbed: nothing here touches a GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_2002_00552_amd/csrc/plan.hpp"

namespace dwm {
dwm_status_t launch_filter_transform(const dwm_plan&, const float*, float*, void*) { return DWM_OK; }
dwm_status_t launch_input_transform(const dwm_plan&, const float*, float*, void*) { return DWM_OK; }
dwm_status_t launch_contract_output(const dwm_plan&, const float*, float*, float*, void*) { return DWM_OK; }
dwm_status_t launch_fused_filter(const dwm_plan&, const float*, float*, void*) { return DWM_OK; }
dwm_status_t launch_fused_forward(const dwm_plan&, const float*, const float*, float*, void*) { return DWM_OK; }
}  // namespace dwm

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd()
{
    g_state ^= g_state << 13;
    g_state ^= g_state >> 7;
    g_state ^= g_state << 17;
    return (uint32_t)(g_state >> 32);
}
static int pick(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }

#define CHECK(c)                                                              \
    do {                                                                      \
        if (!(c)) {                                                           \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); \
            std::exit(2);                                                     \
        }                                                                     \
    } while (0)

static int walk(int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    dwm_plan_t* p = nullptr;
    const dwm_status_t st = dwm_plan_create(&p, N, C, H, W, K, R, S, s, P);
    if (st != DWM_OK) {
        CHECK(p == nullptr);
        CHECK(st == DWM_ERR_INVALID_ARG || st == DWM_ERR_UNSUPPORTED);
        return 0;
    }
    dwm_plan_info_t in;
    CHECK(dwm_plan_info(p, &in) == DWM_OK);
    CHECK(in.OH == (H + 2 * P - R) / s + 1 && in.OW == (W + 2 * P - S) / s + 1);
    CHECK(in.T == (long long)N * in.TH * in.TW);
    // what a launch would ask of a CU: the LDS of the staged input transform and of the single kernel
    CHECK(!p->inlds_ok || (p->inlds.lds_bytes <= 160 * 1024 && p->inlds.cg >= 1 && p->inlds.cg * p->inlds.ncg >= C));
    CHECK(!p->fused_ok || p->fused.lds_bytes <= 160 * 1024);
    // every tap belongs to exactly one part; the multiplication count is the sum over the parts
    std::vector<int> seen((size_t)R * S, 0);
    long long mults = 0;
    for (int i = 0; i < in.n_parts; ++i) {
        dwm_part_t pt;
        CHECK(dwm_plan_part(p, i, &pt) == DWM_OK);
        CHECK(pt.len_h >= 1 && pt.len_h <= 3 && pt.len_w >= 1 && pt.len_w <= 3);
        CHECK(pt.cls >= 0 && pt.cls < in.n_classes);
        mults += (pt.len_h + 1) * (pt.len_w + 1);
        for (int a = 0; a < pt.len_h; ++a)
            for (int b = 0; b < pt.len_w; ++b) {
                const int r = s * (pt.off_h + a) + pt.phase_h, q = s * (pt.off_w + b) + pt.phase_w;
                CHECK(r >= 0 && r < R && q >= 0 && q < S);
                ++seen[(size_t)r * S + q];
            }
    }
    for (int v : seen) CHECK(v == 1);
    CHECK(mults == in.mults_per_tile);
    dwm_part_t bad;
    CHECK(dwm_plan_part(p, in.n_parts, &bad) == DWM_ERR_INVALID_ARG);
    CHECK(dwm_plan_part(p, -1, &bad) == DWM_ERR_INVALID_ARG);
    int planes = 0;
    for (int i = 0; i < in.n_classes; ++i) {
        dwm_class_t c;
        CHECK(dwm_plan_class(p, i, &c) == DWM_OK);
        CHECK(c.L == c.n_parts * C && c.Lpad >= c.L && c.Lpad % 16 == 0);
        planes += (c.len_h + 1) * (c.len_w + 1);
    }
    CHECK(planes == in.n_planes);
    dwm_class_t cbad;
    CHECK(dwm_plan_class(p, in.n_classes, &cbad) == DWM_ERR_INVALID_ARG);
    int nfc, nrows, nslices;
    CHECK(dwm_plan_fused_info(p, &nfc, &nrows, &nslices) == DWM_OK);
    int rows_seen = 0;
    for (int i = 0; i < nfc; ++i) {
        dwm_fused_class_t fc;
        CHECK(dwm_plan_fused_class(p, i, &fc) == DWM_OK);
        CHECK(fc.first_row == rows_seen && fc.rows % 4 == 0);
        rows_seen += fc.rows;
    }
    CHECK(rows_seen == nrows);
    int real_rows = 0;
    for (int r = 0; r < nrows; ++r) {
        dwm_fused_row_t fr;
        CHECK(dwm_plan_fused_row(p, r, &fr) == DWM_OK);
        CHECK(fr.part >= 0 && fr.part < in.n_parts && fr.channel >= 0 && fr.channel < C);
        real_rows += fr.real;
    }
    if (nfc) CHECK(real_rows == in.n_parts * C);
    dwm_fused_row_t frbad;
    CHECK(dwm_plan_fused_row(p, nrows, &frbad) == DWM_ERR_INVALID_ARG);
    // variants: whatever is accepted must leave the sizes sane; nonsense is refused
    static const char* stages[] = {"contract", "split", "input", "input_cg", "forward", "nonsense"};
    for (const char* stage : stages)
        for (int v = -2; v <= 20; ++v) {
            const dwm_status_t sv = dwm_plan_set_variant(p, stage, v);
            CHECK(sv == DWM_OK || sv == DWM_ERR_INVALID_ARG);
            CHECK(dwm_plan_workspace_bytes(p) >= 256 || dwm_plan_workspace_bytes(p) % 4 == 0);
        }
    CHECK(dwm_plan_set_variant(p, "contract", -1) == DWM_OK);
    CHECK(dwm_plan_set_variant(p, "split", 0) == DWM_OK);
    CHECK(dwm_plan_set_variant(p, "forward", -1) == DWM_OK);
    const size_t need = dwm_plan_workspace_bytes(p);
    CHECK(dwm_plan_filter_bytes(p) >= (size_t)4 * in.mults_per_tile * (size_t)C * (size_t)K);
    // the workspace: too small, misaligned, then a (never dereferenced) address that fits
    void* fake = reinterpret_cast<void*>((uintptr_t)1 << 20);
    if (need > 0) CHECK(dwm_plan_set_workspace(p, fake, need - 1) == DWM_ERR_WORKSPACE);
    CHECK(dwm_plan_set_workspace(p, reinterpret_cast<void*>(((uintptr_t)1 << 20) + 4), need) == DWM_ERR_WORKSPACE);
    CHECK(dwm_plan_set_workspace(p, nullptr, need) == DWM_ERR_WORKSPACE);
    float dummy = 0.f;
    CHECK(dwm_conv_forward(p, &dummy, &dummy, &dummy, nullptr) == DWM_ERR_WORKSPACE);
    CHECK(dwm_plan_set_workspace(p, fake, need) == DWM_OK);
    // once the workspace is set its layout is fixed
    CHECK(dwm_plan_set_variant(p, "contract", 10) == DWM_ERR_WORKSPACE);
    CHECK(dwm_plan_set_variant(p, "split", 1) == DWM_ERR_WORKSPACE);
    CHECK(dwm_plan_set_variant(p, "input", 0) == DWM_OK);
    CHECK(dwm_conv_forward(p, &dummy, &dummy, &dummy, nullptr) == DWM_OK);  // the stubs: no launch
    CHECK(dwm_conv_forward(p, nullptr, &dummy, &dummy, nullptr) == DWM_ERR_INVALID_ARG);
    CHECK(dwm_plan_destroy(p) == DWM_OK);
    return 1;
}

// The single-kernel data gradient: its geometry is built on the host (setup.cpp) and the kernel's
// address arithmetic follows from it.  Here that arithmetic is replayed: every LDS offset the
// kernel forms stays inside what it allocates, a staged element is found again where the patch
// reads look for it, and -- on small shapes, in exact integer arithmetic -- the window/tap tables
// give the gradient that the definition gives.
static int walk_bwd_small(int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    using namespace dwm;
    BwdSmallArgs f;
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 0;
    if (H + 2 * P < R || W + 2 * P < S) return 0;
    if (!bwd_small_setup(N, C, H, W, K, R, S, s, P, &f)) return 0;
    const int nfreq = f.four ? 4 : 3, planes = nfreq * nfreq;
    CHECK(f.OH == (H + 2 * P - R) / s + 1 && f.OW == (W + 2 * P - S) / s + 1);
    CHECK(f.nf == C * s * s && f.ncb == (f.nf + 15) / 16);
    // the pieces tile the window, two or three taps each
    int sum = 0;
    for (int i = 0; i < f.nph; ++i) { CHECK(f.jh[i] == sum && (f.lh[i] == 2 || f.lh[i] == 3)); sum += f.lh[i]; }
    CHECK(sum == f.nwh && f.nph <= kBsMaxPieces);
    sum = 0;
    for (int i = 0; i < f.npw; ++i) { CHECK(f.jw[i] == sum && (f.lw[i] == 2 || f.lw[i] == 3)); sum += f.lw[i]; }
    CHECK(sum == f.nww && f.npw <= kBsMaxPieces && f.npp == f.nph * f.npw);
    // every tap of a residue lies inside the window
    for (int rho = 0; rho < s; ++rho) {
        for (int i = 0; i < f.rn_h[rho]; ++i) {
            const int j = f.re_h[rho] + f.Lh - i;
            CHECK(j >= 0 && j < f.nwh && s * i + f.ra_h[rho] < R);
        }
        for (int i = 0; i < f.rn_w[rho]; ++i) {
            const int j = f.re_w[rho] + f.Lw - i;
            CHECK(j >= 0 && j < f.nww && s * i + f.ra_w[rho] < S);
        }
    }
    // tiles and blocks cover the image
    CHECK(2 * s * f.TH >= H && 2 * s * f.TW >= W && f.nbh * f.BH >= f.TH && f.nbw * f.BW >= f.TW && f.BH * f.BW <= 64);
    // LDS: chunks of dy, chunks of the filter copy, the table
    const int G = 1 << f.glog, NE = 1 << f.nelog;
    const long long xs_bytes = 4LL * f.xs_floats, us_bytes = 4LL * f.us_floats;
    const long long pair_bytes = 8LL * f.group_elems, group_bytes = 2 * pair_bytes, row_bytes = 8LL * f.row_elems;
    CHECK((long long)f.lds_bytes == 2 * (xs_bytes + f.nb * us_bytes) + kBsMaxPairs * 8 && f.lds_bytes <= 160 * 1024);
    CHECK(G * group_bytes <= xs_bytes && xs_bytes % 16 == 0 && us_bytes % 1024 == 0);
    CHECK(f.ck == 4 * G && f.steps == f.npp * G && f.steps % 2 == 0 && f.steps >= 2);
    CHECK(f.nchunks * f.ck >= K && (f.nchunks - 1) * f.ck < K);
    CHECK((long long)f.steps * planes * 256 <= us_bytes);
    CHECK(f.nb >= 1 && f.nb <= 3 && f.ncbp >= f.ncb && f.ncbp % f.nb == 0 && f.ncbp < f.ncb + f.nb);
    CHECK(f.u_floats == (size_t)f.ncbp * f.nchunks * f.us_floats);
    CHECK(G * NE <= kBsMaxSlots && f.nrows * f.lw_in <= 256 * NE);
    CHECK(f.row_elems == 2 * f.lwp && f.group_elems == f.nrows * f.row_elems && f.tile_row_step == 2 * f.row_elems);
    // a staged element (r, c) of a channel pair: where the staging writes it; all distinct, all inside
    auto elem_off = [&](int r, int c) { return 8LL * (r * f.row_elems + (c & 1) * f.lwp + (c >> 1)); };
    std::vector<char> used((size_t)(pair_bytes / 8), 0);
    for (int r = 0; r < f.nrows; ++r)
        for (int c = 0; c < f.lw_in; ++c) {
            const long long o = elem_off(r, c);
            CHECK(o >= 0 && o + 8 <= pair_bytes && !used[(size_t)(o / 8)]);
            used[(size_t)(o / 8)] = 1;
        }
    // where a lane looks for patch element (i, j) of piece pair pp: the offsets the kernel adds up
    for (int tl = 0; tl < 64; ++tl) {
        const int by = tl / f.BW, bx = tl % f.BW;
        if (by >= f.BH) continue;
        const long long lane_base = 8LL * (by * f.tile_row_step + bx);
        for (int pp = 0; pp < f.npp; ++pp) {
            const int jh = f.jh[pp / f.npw], jw = f.jw[pp % f.npw];
            for (int i = 0; i < nfreq; ++i)
                for (int j = 0; j < nfreq; ++j) {
                    const long long got = lane_base + ((j & 1) ? f.po1[pp] : f.po0[pp]) + i * row_bytes + (j >> 1) * 8;
                    const int r = 2 * by + jh + i, c = 2 * bx + jw + j;
                    CHECK(r < f.nrows && c < f.lw_in && got == elem_off(r, c));
                }
        }
    }
    // the filter copy: (plane, lane) -> position inside a step is one-to-one
    std::vector<char> upos((size_t)planes * 64, 0);
    for (int pl = 0; pl < planes; ++pl)
        for (int lane = 0; lane < 64; ++lane) {
            const int o = bs_upos(planes, pl, lane);
            CHECK(o >= 0 && o < planes * 64 && !upos[(size_t)o]);
            upos[(size_t)o] = 1;
        }
    // 32-bit offsets: one image of dy, one channel of dx
    CHECK((long long)K * f.OH * f.OW * 4 < (1LL << 31) && (long long)H * W < (1LL << 29));

    // small shapes: the window and tap tables against the definition, in integers
    if ((long long)C * K * H * W * R * S <= 200000 && N <= 2) {
        std::vector<long long> w((size_t)K * C * R * S), dy((size_t)K * f.OH * f.OW);
        for (auto& v : w) v = pick(-3, 3);
        for (auto& v : dy) v = pick(-3, 3);
        for (int c = 0; c < C; ++c)
            for (int ih = 0; ih < H; ++ih)
                for (int iw = 0; iw < W; ++iw) {
                    long long ref = 0;
                    for (int k = 0; k < K; ++k)
                        for (int r = 0; r < R; ++r)
                            for (int q = 0; q < S; ++q) {
                                const int a = ih + P - r, b = iw + P - q;
                                if (a < 0 || b < 0 || a % s || b % s || a / s >= f.OH || b / s >= f.OW) continue;
                                ref += dy[((size_t)k * f.OH + a / s) * f.OW + b / s] * w[(((size_t)k * C + c) * R + r) * S + q];
                            }
                    const int th = ih / s, rh = ih % s, tw = iw / s, rw = iw % s;
                    long long got = 0;
                    for (int k = 0; k < K; ++k)
                        for (int jh = 0; jh < f.nwh; ++jh)
                            for (int jw = 0; jw < f.nww; ++jw) {
                                const int i = f.re_h[rh] + f.Lh - jh, j = f.re_w[rw] + f.Lw - jw;
                                if (i < 0 || i >= f.rn_h[rh] || j < 0 || j >= f.rn_w[rw]) continue;
                                const int a = th - f.Lh + jh, b = tw - f.Lw + jw;
                                if (a < 0 || a >= f.OH || b < 0 || b >= f.OW) continue;
                                got += dy[((size_t)k * f.OH + a) * f.OW + b] *
                                       w[(((size_t)k * C + c) * R + (s * i + f.ra_h[rh])) * S + (s * j + f.ra_w[rw])];
                            }
                    CHECK(got == ref);
                }
    }
    return 1;
}

// The 16-bit single kernel: its geometry (setup.cpp) on the plan cut as eq. 8 prints it.  Every patch
// element a lane reads -- tile base + row entry + row step + column pair -- must be the staged copy of
// the input element the decomposition names, inside the staged region; every padded row must name a
// real (piece, piece, channel); the filter copy must have room for every (class, step, plane, block).
static int walk_fused16(int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    using namespace dwm;
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 0;
    if (H + 2 * P < R || W + 2 * P < S) return 0;
    PlanSpec sp{};
    sp.N = N; sp.C = C; sp.H = H; sp.W = W; sp.K = K; sp.R = R; sp.S = S; sp.stride = s;
    sp.pad_h = sp.pad_w = P;
    sp.OH = (H + 2 * P - R) / s + 1;
    sp.OW = (W + 2 * P - S) / s + 1;
    sp.om = OutMap{sp.OH, sp.OW, 1, 0, 1, 0};
    dwm_plan_t* p = nullptr;
    if (plan_from_spec_as_printed(&p, sp) != DWM_OK) return 0;
    Fused16Args f;
    if (!fused16_setup(*p, &f)) {
        dwm_plan_destroy(p);
        return 0;
    }
    const DevPlan& d = p->d;
    CHECK(f.ncls == d.ncls && f.nkb == (K + 15) / 16 && f.BH * f.BW <= 64 && f.nbh * f.BH >= d.TH && f.nbw * f.BW >= d.TW);
    CHECK(f.row_floats == f.nphase * f.lwp && f.nphase == 2 * s && f.chan_floats == f.nrows * f.row_floats);
    CHECK(f.lds_bytes == (size_t)f.rows_total * 8 + (size_t)C * f.chan_floats * 4 && f.lds_bytes <= 160 * 1024);
    CHECK(f.patch_row_bytes == s * f.row_floats * 4 && f.tile_row_step == 2 * s * f.row_floats);
    auto staged = [&](int r, int c) { return (long long)r * f.row_floats + (c % f.nphase) * f.lwp + c / f.nphase; };
    size_t uf = 0;
    int rows = 0;
    for (int qi = 0; qi < f.ncls; ++qi) {
        const Fused16Class& fc = f.cls[qi];
        const DevClass& q = d.cls[qi];
        CHECK(fc.lh == q.lh && fc.lw == q.lw && fc.L == q.L && fc.row0 == rows && fc.nsteps == (q.L + 15) / 16);
        CHECK((size_t)fc.uf_off == uf);
        uf += (size_t)f.nkb * fc.nsteps * (q.lh + 1) * (q.lw + 1) * 256;
        for (int l = 0; l < 16 * fc.nsteps; ++l, ++rows) {
            const unsigned desc = f.rowdesc[rows];
            const int ph = desc & 15, pw = (desc >> 4) & 15, c = desc >> 8;
            const int lr = l < q.L ? l : q.L - 1;
            const int slot = lr / C;
            CHECK(c == lr % C && ph == q.h0 + slot / q.wn && pw == q.w0 + slot % q.wn);
            CHECK(ph < d.nh && pw < d.nw && d.ph[ph].l == q.lh && d.pw[pw].l == q.lw);
            for (int tl = 0; tl < 64; ++tl) {
                const int by = tl / f.BW, bx = tl % f.BW;
                if (by >= f.BH) continue;
                const long long base = (long long)by * f.tile_row_step + bx + (long long)c * f.chan_floats + f.roff[ph];
                for (int i = 0; i <= q.lh; ++i)
                    for (int j = 0; j <= q.lw; ++j) {
                        const long long got = base + (long long)i * (f.patch_row_bytes / 4) + ((j & 1) ? f.coff1[pw] : f.coff0[pw]) + (j >> 1);
                        const int r = 2 * s * by + s * (d.ph[ph].j + i) + d.ph[ph].p;
                        const int cc = 2 * s * bx + s * (d.pw[pw].j + j) + d.pw[pw].p;
                        CHECK(r < f.nrows && cc < f.lw_in);
                        CHECK(got == (long long)c * f.chan_floats + staged(r, cc));
                        CHECK(got >= 0 && (got + 1) * 4 <= (long long)C * f.chan_floats * 4);
                    }
            }
        }
    }
    CHECK(rows == f.rows_total && uf == f.uf_halves && rows <= kF16MaxRows);
    CHECK((long long)K * d.OH * d.OW * 4 < (1LL << 31) && uf * 2 < ((size_t)1 << 31));
    dwm_plan_destroy(p);
    return 1;
}

int main(int argc, char** argv)
{
    const int iters = argc > 1 ? std::atoi(argv[1]) : 3000;
    int ok = 0, tried = 0, small = 0, single16 = 0;
    // the benchmark layers and corner shapes first
    const int fixed[][9] = {
        {1, 16, 32, 32, 16, 5, 5, 1, 2},   {32, 128, 56, 56, 256, 3, 3, 2, 1}, {32, 256, 28, 28, 256, 7, 7, 1, 3},
        {64, 3, 224, 224, 64, 7, 7, 2, 3}, {128, 3, 227, 227, 96, 11, 11, 4, 0}, {1, 1, 1, 1, 1, 1, 1, 1, 0},
        {1, 1, 48, 48, 1, 48, 48, 1, 0},   {1, 1, 49, 49, 1, 49, 49, 1, 0},      {1, 1, 7, 7, 1, 1, 1, 9, 0},
        {1, 1, 3, 3, 1, 5, 5, 1, 0},       {0, 1, 3, 3, 1, 3, 3, 1, 0},          {1, 1, 3, 3, 1, 3, 3, 0, 0},
        {1, 1, 3, 3, 1, 3, 3, 1, -1},      {1, 127, 64, 64, 1, 3, 3, 1, 1},      {1, 128, 64, 64, 1, 3, 3, 1, 1},
        {1, 1, 1 << 20, 2, 1, 3, 1, 1, 1}, {1, 1, 2, (1 << 20) + 1, 1, 1, 3, 1, 1}, {4096, 1, 1024, 1024, 1, 3, 3, 1, 1},
        {1, 2, 12, 6000, 3, 3, 3, 1, 1},   {1, 3, 300, 300, 8, 33, 3, 16, 5},    {2, 5, 40, 40, 33, 47, 47, 1, 23},
        {6, 12, 68, 10, 116, 10, 10, 4, 3},  // one tile per row: a block of 64 tiles spans whole images (45 KB a channel)
    };
    for (const auto& f : fixed) {
        ++tried;
        ok += walk(f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[7], f[8]);
        small += walk_bwd_small(f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[7], f[8]);
        single16 += walk_fused16(f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[7], f[8]);
    }
    // the contraction the planner picks: the three-stage ring of 32-row chunks (11) for three rounds of tiles and for
    // long reductions above one tile per CU, the two-stage ring of 64-row chunks (12) otherwise
    {
        const int pinned[][10] = {
            {32, 256, 28, 28, 256, 7, 7, 1, 3, 11},   // 392 tiles of 25 600 rows
            {32, 128, 56, 56, 256, 3, 3, 2, 1, 12},   // 392 tiles of 3200 rows
            {16, 256, 28, 28, 256, 7, 7, 1, 3, 12},   // 196 tiles: every tile cut into ranges of its own
            {64, 256, 28, 28, 256, 3, 3, 1, 1, 11},   // 784 tiles: three rounds
            {8, 64, 28, 28, 64, 3, 3, 1, 1, 12},      // 25 tiles of short reductions
        };
        for (const auto& f : pinned) {
            dwm_plan_t* p = nullptr;
            CHECK(dwm_plan_create(&p, f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[7], f[8]) == DWM_OK);
            CHECK(p->geo.variant == f[9]);
            CHECK(dwm_plan_destroy(p) == DWM_OK);
        }
    }
    CHECK(dwm_plan_create(nullptr, 1, 1, 3, 3, 1, 3, 3, 1, 1) == DWM_ERR_INVALID_ARG);
    CHECK(dwm_plan_destroy(nullptr) == DWM_ERR_INVALID_ARG);
    CHECK(dwm_plan_filter_bytes(nullptr) == 0 && dwm_plan_workspace_bytes(nullptr) == 0);
    for (int it = 0; it < iters; ++it) {
        const int R = pick(1, 13), S = pick(1, 13), s = pick(1, 5), P = pick(0, 6);
        const int big = rnd() % 8 == 0;
        const int H = pick(1, big ? 400 : 40), W = pick(1, big ? 400 : 40);
        const int C = pick(1, rnd() % 4 == 0 ? 300 : 20), K = pick(1, rnd() % 4 == 0 ? 300 : 40);
        const int N = pick(1, big ? 3 : 70);
        ++tried;
        ok += walk(N, C, H, W, K, R, S, s, P);
        small += walk_bwd_small(N, C < 20 ? C : C % 9 + 1, H, W, K, R, S, s, P);
        single16 += walk_fused16(N, C < 20 ? C : C % 9 + 1, H, W, K, R, S, s, P);
    }
    CHECK(small > tried / 8 && single16 > tried / 8);
    std::printf("planner fuzz: %d shapes tried, %d planned, %d with a single-kernel data gradient, %d with a 16-bit single kernel\n",
                tried, ok, small, single16);
    return ok > tried / 2 ? 0 : 3;
}
