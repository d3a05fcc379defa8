// Host-side geometry of two kernels of libdwm: which block of tiles a workgroup of the
// single-kernel forward path owns and how its input region is staged in LDS (fused.hip), and how
// the LDS-staged input transform stages its rows (transforms.hip).  Pure integer logic, no GPU
// call: this file and plan.cpp also build with a plain host compiler (sanitizer builds).
#include <algorithm>

#include "plan.hpp"

namespace dwm {

// ---------------------------------------------------------------------------------
// Single-kernel forward path: does it apply, and with which block of tiles
// ---------------------------------------------------------------------------------
bool fused_setup(const dwm_plan& p, FusedArgs* out)
{
    const DevPlan& d = p.d;
    FusedArgs f{};
    if (d.C > 127 || d.nh > 15 || d.nw > 15) return false;
    // classes = pairs of families; inside a class the rows (part, channel) follow each other sorted by
    // (len_h, len_w), longest first, and only the class's end is padded to a multiple of four.  A step
    // whose four rows mix piece lengths runs the planes of the longest: the shorter pieces' rows hold
    // zeros in the filter copy for the frequencies they lack.
    int rows = 0, steps = 0;
    int row_lh[kFusedMaxRows], row_lw[kFusedMaxRows];
    for (int wh = 1; wh >= 0; --wh)
        for (int ww = 1; ww >= 0; --ww) {
            FusedClass fc{};
            fc.wide_h = wh; fc.wide_w = ww;
            fc.nfh = wh ? 4 : 2; fc.nfw = ww ? 4 : 2;
            fc.step0 = steps; fc.row0 = rows;
            for (int lh = 3; lh >= 1; --lh)
                for (int lw = 3; lw >= 1; --lw) {
                    if ((lh >= 2) != (wh == 1) || (lw >= 2) != (ww == 1)) continue;
                    for (int a = 0; a < d.nh; ++a)
                        for (int b = 0; b < d.nw; ++b) {
                            if (d.ph[a].l != lh || d.pw[b].l != lw) continue;
                            for (int c = 0; c < d.C; ++c) {
                                if (rows >= kFusedMaxRows) return false;
                                f.rowdesc[rows] = (unsigned short)(a | b << 4 | c << 8 | 1 << 15);
                                row_lh[rows] = lh; row_lw[rows] = lw;
                                ++rows;
                            }
                        }
                }
            if (rows == fc.row0) continue;
            while ((rows - fc.row0) & 3) {  // padding rows: a real row's offsets, zero filter rows
                if (rows >= kFusedMaxRows) return false;
                f.rowdesc[rows] = (unsigned short)(f.rowdesc[rows - 1] & 0x7fff);
                row_lh[rows] = row_lh[rows - 1]; row_lw[rows] = row_lw[rows - 1];
                ++rows;
            }
            for (int r0 = fc.row0; r0 < rows; r0 += 4) {
                if (steps >= kFusedMaxSteps) return false;
                int mh = 0, mw = 0;
                for (int r = r0; r < r0 + 4; ++r) { mh = std::max(mh, row_lh[r]); mw = std::max(mw, row_lw[r]); }
                f.step_type[steps++] = mh * 4 + mw;
            }
            fc.nsteps = steps - fc.step0;
            fc.rows = rows - fc.row0;
            f.fc[f.nfc++] = fc;
        }
    f.rows_total = rows;

    // One class of two- and three-tap pieces only: the kernel then reads a patch row
    // as two pairs of adjacent LDS words (columns 0,2 and 1,3 of the patch lie 2*stride input columns
    // apart, i.e. one word apart in the de-interleaved row), also for two-tap pieces, whose fourth
    // column is then the input's real next element (it only meets zeros of the filter copy): the
    // staged region is as wide as if every piece had three taps.
    f.wide = f.nfc == 1 && f.fc[0].wide_h && f.fc[0].wide_w;
    int max_oh = 0, max_ow = 0;
    for (int i = 0; i < d.nh; ++i) max_oh = std::max(max_oh, d.s * (d.ph[i].j + d.ph[i].l) + d.ph[i].p);
    for (int i = 0; i < d.nw; ++i) max_ow = std::max(max_ow, d.s * (d.pw[i].j + (f.wide ? 3 : d.pw[i].l)) + d.pw[i].p);
    f.nphase = 2 * d.s;
    const size_t table_bytes = (size_t)rows * 64;
    const size_t budget = 72 * 1024;  // two workgroups per CU

    // block of tiles: most useful lanes first, then the smallest staged region
    double best_eff = 0.0;
    size_t best_x = 0;
    for (int bw = 1; bw <= 64 && bw <= d.TW; ++bw) {
        int bh = 64 / bw;
        if (bh > d.TH) bh = d.TH;
        if (bh < 1) continue;
        const int nbh = (d.TH + bh - 1) / bh, nbw = (d.TW + bw - 1) / bw;
        const double eff = (double)d.TH * d.TW / ((double)nbh * nbw * 64);
        const long long nrows = 2LL * d.s * (bh - 1) + max_oh + 1;
        const long long lw_in = 2LL * d.s * (bw - 1) + max_ow + 1;
        const long long lwp = ((lw_in + f.nphase - 1) / f.nphase) | 1;
        const long long x_bytes = (long long)d.C * nrows * f.nphase * lwp * (long long)sizeof(float);
        if (x_bytes + (long long)table_bytes > (long long)budget) continue;
        if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && (size_t)x_bytes < best_x)) {
            best_eff = eff; best_x = (size_t)x_bytes;
            f.BH = bh; f.BW = bw; f.nbh = nbh; f.nbw = nbw;
            f.nrows = (int)nrows; f.lw_in = (int)lw_in; f.lwp = (int)lwp;
        }
    }
    if (best_eff < 0.5) return false;
    const long long blocks = (long long)d.N * f.nbh * f.nbw;
    if (blocks > 0x7fffffffLL) return false;
    f.row_floats = f.nphase * f.lwp;
    f.chan_floats = f.nrows * f.row_floats;
    f.tile_row_step = 2 * d.s * f.row_floats;
    f.nslices = (d.K + 31) / 32;
    // with few blocks the filter slices are spread over workgroups as well
    f.slices_per_wg = blocks >= 2 * kNumCUs ? f.nslices : 1;
    f.nkw = (f.nslices + f.slices_per_wg - 1) / f.slices_per_wg;
    if (f.nkw > 65535) return false;
    f.div_bw.init((unsigned)f.BW);
    f.div_nphase.init((unsigned)f.nphase);
    for (int i = 0; i < kMaxPieces; ++i)
        for (int k = 0; k < 4; ++k) {
            // offsets past a piece's own patch (k > its length) repeat its last element: they are read
            // (the patch is always read 4 wide) and only ever multiplied by zeros, but must be finite
            // (with a single class of two- and three-tap pieces the real fourth column is read instead: see above)
            const int kh = i < d.nh ? std::min(k, d.ph[i].l) : 0, kw = i < d.nw ? (f.wide ? k : std::min(k, d.pw[i].l)) : 0;
            const int oh = i < d.nh ? d.s * (d.ph[i].j + kh) + d.ph[i].p : 0;
            const int ow = i < d.nw ? d.s * (d.pw[i].j + kw) + d.pw[i].p : 0;
            f.roff[i][k] = oh * f.row_floats;
            f.coff[i][k] = (ow % f.nphase) * f.lwp + ow / f.nphase;
        }
    for (int i = 0; i < d.nw; ++i)  // columns two apart are one word apart in a de-interleaved row
        if (f.wide && (f.coff[i][2] != f.coff[i][0] + 1 || f.coff[i][3] != f.coff[i][1] + 1)) return false;
    f.lds_bytes = table_bytes + best_x;
    *out = f;
    return true;
}


// Does the LDS-staged form apply, and with how many channels per workgroup: the rows a block
// stages must fit in LDS.  The row count depends on where a block of 64 tiles starts; the
// pattern repeats after at most TH*TW blocks, so the maximum is found by walking them.
bool input_lds_setup(const dwm_plan& p, InLdsArgs* out, int cg_wish)
{
    const DevPlan& d = p.d;
    InLdsArgs a{};
    int max_oh = 0, max_ow = 0;
    for (int i = 0; i < d.nh; ++i) max_oh = std::max(max_oh, d.s * (d.ph[i].j + d.ph[i].l) + d.ph[i].p);
    for (int i = 0; i < d.nw; ++i) max_ow = std::max(max_ow, d.s * (d.pw[i].j + d.pw[i].l) + d.pw[i].p);
    if (d.s > 4096 || max_oh > (1 << 20) || max_ow > (1 << 20)) return false;
    a.nphase = 2 * d.s;
    a.foot_h = max_oh + 1;
    const long long lw_in = 2LL * d.s * (d.TW - 1) + max_ow + 1;
    const long long rows_full = 2LL * d.s * (d.TH - 1) + a.foot_h;
    if (lw_in > (1 << 16) || rows_full > (1 << 24)) return false;
    a.lw_in = (int)lw_in;
    a.lwp = ((a.lw_in + a.nphase - 1) / a.nphase) | 1;
    a.row_floats = a.nphase * a.lwp;
    a.rows_full = (int)rows_full;
    const long long per = (long long)d.TH * d.TW;
    const long long nb = (d.T + 63) / 64, scan = std::min(nb, per);
    long long max_rows = 0;
    const int s2 = 2 * d.s;
    for (long long bt = 0; bt < scan; ++bt) {
        const long long t0 = bt * 64, t1 = std::min<long long>(t0 + 63, d.T - 1);
        const long long g0 = t0 / d.TW, g1 = t1 / d.TW, n0 = g0 / d.TH, n1 = g1 / d.TH;
        const long long ty_a0 = g0 - n0 * d.TH, ty_b1 = g1 - n1 * d.TH;
        const long long rows0 = s2 * ((n1 == n0 ? ty_b1 : d.TH - 1) - ty_a0) + a.foot_h;
        const long long total = n1 == n0 ? rows0 : rows0 + (n1 - n0 - 1) * rows_full + s2 * ty_b1 + a.foot_h;
        max_rows = std::max(max_rows, total);
        if (max_rows * a.row_floats * 4 > 64 * 1024) return false;
    }
    a.max_rows = (int)max_rows;
    a.chan_floats = a.max_rows * a.row_floats;
    const size_t chan_bytes = (size_t)a.chan_floats * sizeof(float);
    if (chan_bytes > 64 * 1024) return false;
    // channels per workgroup: one per wave (measured best: many small workgroups keep more loads
    // and stores in flight than fewer large ones)
    int cg = d.C < 4 ? d.C : 4;
    while (cg > 1 && cg * chan_bytes > 150 * 1024) --cg;  // (a channel's region fits by the check above)
    if (cg_wish > 0 && cg_wish <= d.C && cg_wish * chan_bytes <= 150 * 1024) cg = cg_wish;
    a.cg = cg;
    a.ncg = (d.C + cg - 1) / cg;
    if ((long long)a.ncg * (d.Tpad / 64) > 0x7fffffffLL) return false;
    a.div_tw.init((unsigned)d.TW);
    a.div_th.init((unsigned)d.TH);
    a.div_lw.init((unsigned)a.lw_in);
    a.div_nphase.init((unsigned)a.nphase);
    a.div_rows_full.init((unsigned)a.rows_full);
    for (int i = 0; i < kMaxPieces; ++i)
        for (int k = 0; k < 4; ++k) {
            const int oh = i < d.nh ? d.s * (d.ph[i].j + k) + d.ph[i].p : 0;
            const int ow = i < d.nw ? d.s * (d.pw[i].j + k) + d.pw[i].p : 0;
            a.roff[i][k] = oh * a.row_floats;
            a.coff[i][k] = (ow % a.nphase) * a.lwp + ow / a.nphase;
        }
    a.lds_bytes = (size_t)cg * chan_bytes;
    *out = a;
    return true;
}

// ---------------------------------------------------------------------------------
// Single-kernel data gradient (few input channels): window, pieces, block of tiles, LDS
// ---------------------------------------------------------------------------------
// One dimension: residues of the dx coordinate modulo the stride, the common window of dy and
// its cut into pieces of three and two taps (3,...,3 then 2 or 2,2: never a single tap).
static bool bwd_small_dim(int R, int s, int P, int* ra, int* re, int* rn, int* L, int* nwin, int* np, int* pj, int* pl)
{
    bool any = false;
    int lmax = 0, emax = 0;
    for (int rho = 0; rho < s; ++rho) {
        const int a = (rho + P) % s, e = (rho + P) / s;
        const int n = a < R ? (R - a + s - 1) / s : 0;
        ra[rho] = a; re[rho] = e; rn[rho] = n;
        if (n == 0) continue;
        if (!any || n - 1 - e > lmax) lmax = n - 1 - e;
        if (!any || e > emax) emax = e;
        any = true;
    }
    if (!any) return false;
    *L = lmax;
    const int n = emax + lmax + 1;
    *nwin = n;
    if (n < 2 || n > 11) return false;
    int cnt = 0, j = 0, left = n;
    while (left > 0) {
        const int l = (left == 2 || left == 4) ? 2 : 3;
        if (cnt >= kBsMaxPieces) return false;
        pj[cnt] = j; pl[cnt] = l;
        ++cnt; j += l; left -= l;
    }
    *np = cnt;
    return true;
}

bool bwd_small_setup(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, BwdSmallArgs* out)
{
    BwdSmallArgs f{};
    const int s = stride;
    if (s < 1 || s > 8 || N < 1 || C < 1 || K < 1 || pad < 0 || pad > (1 << 20) || H > (1 << 20) || W > (1 << 20)) return false;
    f.N = N; f.C = C; f.H = H; f.W = W; f.K = K; f.s = s;
    f.OH = (H + 2 * pad - R) / s + 1;
    f.OW = (W + 2 * pad - S) / s + 1;
    if (f.OH < 1 || f.OW < 1) return false;
    // one image of dy is addressed through a 32-bit buffer offset, dx through 32-bit pixel offsets
    if ((long long)K * f.OH * f.OW * 4 >= (1LL << 31) || (long long)H * W >= (1LL << 29)) return false;
    const long long nf = (long long)C * s * s;
    if (nf > 256) return false;
    f.nf = (int)nf;
    f.ncb = (f.nf + 15) / 16;
    // column blocks a wave accumulates in one pass over dy: the fewest passes, then the fewest blocks per pass
    f.nb = 1;
    for (int nb = 2; nb <= 3; ++nb)
        if ((f.ncb + nb - 1) / nb < (f.ncb + f.nb - 1) / f.nb) f.nb = nb;
    f.ncbp = (f.ncb + f.nb - 1) / f.nb * f.nb;
    if (!bwd_small_dim(R, s, pad, f.ra_h, f.re_h, f.rn_h, &f.Lh, &f.nwh, &f.nph, f.jh, f.lh)) return false;
    if (!bwd_small_dim(S, s, pad, f.ra_w, f.re_w, f.rn_w, &f.Lw, &f.nww, &f.npw, f.jw, f.lw)) return false;
    f.npp = f.nph * f.npw;
    f.four = 0;
    for (int i = 0; i < f.nph; ++i) f.four |= f.lh[i] == 3;
    for (int i = 0; i < f.npw; ++i) f.four |= f.lw[i] == 3;
    const int nfreq = f.four ? 4 : 3, planes = nfreq * nfreq;
    const int th = (H + s - 1) / s, tw = (W + s - 1) / s;  // window positions per dimension
    f.TH = (th + 1) / 2; f.TW = (tw + 1) / 2;
    // the patch of a piece is read nfreq wide whatever its length
    const int max_oh = f.jh[f.nph - 1] + nfreq - 1, max_ow = f.jw[f.npw - 1] + nfreq - 1;
    // Bank conflicts of a patch read: LDS serves 32 lanes a cycle from 32 banks of four bytes.  A group of
    // four channels is staged as two planes of channel pairs, [element][2]; the lanes of half a wave are
    // 16 tiles x the two channels of one pair and read word 2*(element of the tile) + (channel & 1).
    // Returns the worst multiplicity of a bank over the four waves.
    auto conflicts = [&](int bw, int bh, int lwp) {
        int worst = 0;
        for (int wave = 0; wave < 4; ++wave) {
            int cnt[32] = {0};
            for (int n = 0; n < 16; ++n) {
                const int tl = wave * 16 + n, by = tl / bw, bx = tl % bw;
                const int el = by < bh ? by * 4 * lwp + bx : 0;
                for (int q = 0; q < 2; ++q) worst = std::max(worst, ++cnt[(2 * el + q) & 31]);
            }
        }
        return worst;
    };
    // block of tiles: most useful lanes first, then the cheapest staged region; the chunk of channels is the
    // largest (8, 16 or 32) with which two workgroups fit a CU, else 8
    double best_eff = 0.0;
    long long best_x = 0, best_cost = 0;
    for (int bw = 1; bw <= 64 && bw <= f.TW; ++bw) {
        int bh = 64 / bw;
        if (bh > f.TH) bh = f.TH;
        if (bh < 1) continue;
        const int nbh = (f.TH + bh - 1) / bh, nbw = (f.TW + bw - 1) / bw;
        const double eff = (double)f.TH * f.TW / ((double)nbh * nbw * 64);
        const long long nrows = 2LL * (bh - 1) + max_oh + 1;
        const long long lw_in = 2LL * (bw - 1) + max_ow + 1;
        if (nrows * lw_in > 256LL * kBsMaxSlots / 2) continue;
        int nelog = 0;
        while ((256LL << nelog) < nrows * lw_in) ++nelog;
        // the largest chunk first; for it, the row padding with the fewest bank conflicts that still fits
        const long long lwp0 = (lw_in + 1) / 2;
        long long lwp = lwp0, group = 0;
        int glog = -1;
        // (nine planes leave registers for three waves per SIMD: three workgroups per CU, 52 KB each;
        // sixteen planes: two, 79 KB each; with several column blocks per wave two and one, 79 and 150 KB;
        // a chunk of four channels only with an even number of steps)
        const int wg_kb = f.nb > 1 ? (f.four ? 150 : 79) : (f.four ? 79 : 52);
        for (int g = 3; g >= 0 && glog < 0; --g) {
            if ((1 << g) << nelog > kBsMaxSlots || ((f.npp << g) & 1)) continue;
            const long long us = ((long long)(f.npp << g) * planes * 64 + 255) / 256 * 256;
            int best_c = 1 << 30;
            for (long long l = lwp0; l < lwp0 + 4; ++l) {
                const long long grp = nrows * 2 * l;  // elements of four floats
                const long long bytes = 2 * ((grp << g) * 4 + f.nb * us) * (long long)sizeof(float);
                if (bytes > (g > (f.npp & 1) ? wg_kb : 150) * 1024) continue;
                const int c = conflicts(bw, bh, (int)l);
                if (c < best_c) { best_c = c; lwp = l; group = grp; glog = g; }
            }
        }
        if (glog < 0) continue;
        const long long xs = (group << glog) * 4;
        // among equally full blocks: the least to load, a row of the region counted 16 elements longer than
        // it is (short rows waste most of the memory transactions that fetch them)
        const long long cost = nrows * (lw_in + 16);
        if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && cost < best_cost)) {
            best_eff = eff; best_x = xs; best_cost = cost;
            f.BH = bh; f.BW = bw; f.nbh = nbh; f.nbw = nbw;
            f.nrows = (int)nrows; f.lw_in = (int)lw_in; f.lwp = (int)lwp;
            f.glog = glog; f.nelog = nelog;
        }
    }
    if (best_eff <= 0.0) return false;
    f.eff_pct = (int)(best_eff * 100.0);
    if ((long long)N * f.nbh * f.nbw > 0x7fffffffLL) return false;
    f.ck = 4 << f.glog;
    f.steps = f.npp << f.glog;
    f.nchunks = (K + f.ck - 1) / f.ck;
    f.us_floats = (f.steps * planes * 64 + 255) / 256 * 256;  // whole 1 KB pieces: one DMA instruction of a wave each
    f.row_elems = 2 * f.lwp;
    f.group_elems = f.nrows * f.row_elems;
    f.tile_row_step = 2 * f.row_elems;
    f.xs_floats = (int)best_x;
    f.div_bw.init((unsigned)f.BW);
    f.div_lw.init((unsigned)f.lw_in);
    for (int pp = 0; pp < f.npp; ++pp) {
        const int jh = f.jh[pp / f.npw], jw = f.jw[pp % f.npw];
        f.po0[pp] = 8 * (jh * f.row_elems + (jw & 1) * f.lwp + (jw >> 1));
        f.po1[pp] = 8 * (jh * f.row_elems + ((jw + 1) & 1) * f.lwp + ((jw + 1) >> 1));
    }
    // LDS: two staged chunks of dy, two chunks of the filter copy, the table of patch offsets
    f.lds_bytes = 2 * ((size_t)f.xs_floats + (size_t)f.nb * f.us_floats) * sizeof(float) + kBsMaxPairs * 8;
    f.u_floats = (size_t)f.ncbp * f.nchunks * f.us_floats;
    *out = f;
    return true;
}

// ---------------------------------------------------------------------------------
// 16-bit single-kernel forward path: classes, rows, block of tiles, LDS
// ---------------------------------------------------------------------------------
bool fused16_setup(const dwm_plan& p, Fused16Args* out)
{
    const DevPlan& d = p.d;
    Fused16Args f{};
    if (d.C > 127 || d.nh > 15 || d.nw > 15 || d.ncls > kMaxClasses) return false;
    if (d.om.sy != 1 || d.om.sx != 1 || d.om.oy != 0 || d.om.ox != 0 || d.om.YH != d.OH || d.om.YW != d.OW) return false;
    f.nkb = (d.K + 15) / 16;
    f.slice_kb = std::min(f.nkb, 2);  // (the launcher sets what its kernel takes)
    f.nslices = (f.nkb + f.slice_kb - 1) / f.slice_kb;
    int rows = 0;
    size_t uf = 0;
    for (int qi = 0; qi < d.ncls; ++qi) {
        const DevClass& q = d.cls[qi];
        Fused16Class fc{};
        fc.lh = q.lh; fc.lw = q.lw;
        fc.L = q.L;
        fc.row0 = rows;
        fc.nsteps = (q.L + 15) / 16;
        fc.uf_off = (long long)uf;
        for (int l = 0; l < fc.nsteps * 16; ++l) {
            if (rows >= kF16MaxRows) return false;
            const int lr = std::min(l, q.L - 1);  // padding rows: the last real row's patch, zero filter rows
            const int slot = lr / d.C, c = lr - slot * d.C;
            const int a = slot / q.wn, b = slot - a * q.wn;
            f.rowdesc[rows++] = (unsigned short)((q.h0 + a) | (q.w0 + b) << 4 | c << 8);
        }
        uf += (size_t)f.nkb * fc.nsteps * (q.lh + 1) * (q.lw + 1) * 256;
        f.cls[f.ncls++] = fc;
    }
    f.rows_total = rows;
    f.uf_halves = uf;
    if (uf * 2 >= ((size_t)1 << 31)) return false;  // addressed through a 32-bit buffer offset
    if ((long long)d.K * d.OH * d.OW * 4 >= (1LL << 31)) return false;  // ... and so is one image of y

    int max_oh = 0, max_ow = 0;
    for (int i = 0; i < d.nh; ++i) max_oh = std::max(max_oh, d.s * (d.ph[i].j + d.ph[i].l) + d.ph[i].p);
    for (int i = 0; i < d.nw; ++i) max_ow = std::max(max_ow, d.s * (d.pw[i].j + d.pw[i].l) + d.pw[i].p);
    f.nphase = 2 * d.s;
    const size_t table_bytes = (size_t)rows * 8;
    const size_t budget = 76 * 1024;  // two workgroups per CU
    double best_eff = 0.0;
    size_t best_x = 0;
    for (int bw = 1; bw <= 64 && bw <= d.TW; ++bw) {
        int bh = 64 / bw;
        if (bh > d.TH) bh = d.TH;
        if (bh < 1) continue;
        const int nbh = (d.TH + bh - 1) / bh, nbw = (d.TW + bw - 1) / bw;
        const double eff = (double)d.TH * d.TW / ((double)nbh * nbw * 64);
        const long long nrows = 2LL * d.s * (bh - 1) + max_oh + 1;
        const long long lw_in = 2LL * d.s * (bw - 1) + max_ow + 1;
        const long long lwp = ((lw_in + f.nphase - 1) / f.nphase) | 1;
        const long long x_bytes = (long long)d.C * nrows * f.nphase * lwp * (long long)sizeof(float);
        if (x_bytes + (long long)table_bytes > (long long)budget) continue;
        if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && (size_t)x_bytes < best_x)) {
            best_eff = eff; best_x = (size_t)x_bytes;
            f.BH = bh; f.BW = bw; f.nbh = nbh; f.nbw = nbw;
            f.nrows = (int)nrows; f.lw_in = (int)lw_in; f.lwp = (int)lwp;
        }
    }
    if (best_eff <= 0.0) return false;
    f.eff_pct = (int)(best_eff * 100.0);
    if ((long long)d.N * f.nbh * f.nbw > 0x7fffffffLL) return false;
    f.row_floats = f.nphase * f.lwp;
    f.chan_floats = f.nrows * f.row_floats;
    f.tile_row_step = 2 * d.s * f.row_floats;
    f.patch_row_bytes = d.s * f.row_floats * 4;
    f.div_bw.init((unsigned)f.BW);
    f.div_nphase.init((unsigned)f.nphase);
    for (int i = 0; i < kMaxPieces; ++i) {
        const int oh = i < d.nh ? d.s * d.ph[i].j + d.ph[i].p : 0;
        const int ow0 = i < d.nw ? d.s * d.pw[i].j + d.pw[i].p : 0, ow1 = ow0 + d.s;
        f.roff[i] = oh * f.row_floats;
        f.coff0[i] = (ow0 % f.nphase) * f.lwp + ow0 / f.nphase;
        f.coff1[i] = (ow1 % f.nphase) * f.lwp + ow1 / f.nphase;
    }
    f.lds_bytes = table_bytes + best_x;
    *out = f;
    return true;
}

}  // namespace dwm
