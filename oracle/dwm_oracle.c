/*
 * FP64 CPU oracle for the Decomposable Winograd Method (DWM) forward convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or call
 * this file; it exists so that tests, the smoke check and the benchmark's CPU
 * baseline leg have an independent statement of what the GPU path must compute.
 * It shares no code, tables or helpers with the HIP library.
 *
 * Two independent computations of the same result:
 *
 *   O1  oracle_direct_f64      the plain definition of a strided, zero-padded 2-D
 *                              cross-correlation (what the paper calls "regular
 *                              convolution"; its aggregation step states that DWM's
 *                              result is equal to it, Sec. 4.1 "Aggregation").
 *   O2  oracle_dwm_f64         the paper's five steps, in its order (Sec. 4.1 bullet
 *                              list, Fig. 3): splitting, transformation, calculation,
 *                              detransformation, aggregation; stride handled by the
 *                              phase grouping of Sec. 4.1 "Stride > 1" (eq. 12-14),
 *                              size by the consecutive 3-tap cut of Sec. 4.1 "Large
 *                              kernel size" (eq. 8-11).
 *
 *   O2h oracle_dwm_half_f64    O2 with half-precision storage (the "DWM FP16" column of
 *                              Table 1): x and w hold binary16 values, the transformed
 *                              filter U and the transformed input V are rounded to
 *                              binary16 (nearest, ties to even) before they are
 *                              multiplied; every sum is FP64 and the result is returned
 *                              unrounded.  The paper does not say where its FP16
 *                              implementation rounds; this reading is the one a matrix
 *                              unit with FP16 operands and a wide accumulator computes.
 *                              U is rounded from its exact value; V from B^T d B evaluated in
 *                              binary32, columns first (part_input_transform_binary32): the
 *                              precision in which the 16-bit value of an element is decided
 *                              is part of the reading, and binary32 is what such a path
 *                              transforms in (exact for all but sums spanning 13+ binades).
 *   O2b oracle_dwm_bf16_f64    the same reading with bfloat16 storage (8 significant bits,
 *                              binary32's exponent range): the other 16-bit format such
 *                              matrix units take.
 *
 * and, for the gradient with respect to the input (the paper's backward pass, Sec. 3.1
 * eq. 5 and Sec. 4.2 eq. 16-17):
 *
 *   O1' oracle_backward_data_f64      the definition of dL/dx
 *   O2' oracle_dwm_backward_data_f64  the paper's formulas, part by part
 * and for the gradient with respect to the filter (Sec. 3.1 eq. 5, Sec. 4.2 eq. 18):
 *   O1'' oracle_backward_filter_f64, O2'' oracle_dwm_backward_filter_f64
 *
 * All arithmetic is double precision; inputs are the float32 arrays the GPU sees,
 * widened on load.  Layouts: x[N][C][H][W], w[K][C][R][S], y[N][K][OH][OW], dense.
 * Cross-correlation semantics (the printed F(2,3) matrices of Sec. 3.2 compute
 * y_j = sum_k d_{j+k} g_k): y[n,k,oh,ow] = sum_{c,r,q} xp[n,c,oh*s+r,ow*s+q] w[k,c,r,q],
 * xp = x zero-padded by P on all four sides.
 *
 * Pins: see tests/test_oracle_*.py (rational-arithmetic identity of every F(2,l),
 * the printed F(2,3) matrices, Table 3 multiplication counts, closed forms, a
 * library float64 convolution, brute force, and O2 == O1 to 1e-12).
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* O1: direct convolution, the definition                                     */
/* ------------------------------------------------------------------------- */

static double direct_point(const float* x, const float* w, int C, int H, int W,
                           int R, int S, int s, int P, int n, int k, int oh, int ow)
{
    double acc = 0.0;
    for (int c = 0; c < C; ++c)
        for (int r = 0; r < R; ++r)
            for (int q = 0; q < S; ++q) {
                int ih = oh * s + r - P;
                int iw = ow * s + q - P;
                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue; /* zero padding */
                double xv = (double)x[(((size_t)n * C + c) * H + ih) * W + iw];
                double wv = (double)w[(((size_t)k * C + c) * R + r) * S + q];
                acc += xv * wv;
            }
    return acc;
}

int oracle_out_size(int H, int R, int s, int P) { return (H + 2 * P - R) / s + 1; }

/* y[N][K][OH][OW] <- direct convolution.  Returns 0, or 1 on a bad shape. */
int oracle_direct_f64(const float* x, const float* w, double* y,
                      int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = oracle_out_size(H, R, s, P), OW = oracle_out_size(W, S, s, P);
    const long long NK = (long long)N * K;
#pragma omp parallel for schedule(dynamic, 1)
    for (long long nk = 0; nk < NK; ++nk) {
        int n = (int)(nk / K), k = (int)(nk % K);
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow)
                y[(((size_t)n * K + k) * OH + oh) * OW + ow] =
                    direct_point(x, w, C, H, W, R, S, s, P, n, k, oh, ow);
    }
    return 0;
}

/* out[i] <- y at flat output index idx[i] (index into [N][K][OH][OW]); for sampled
 * checks at sizes where the whole output is too slow to compute. */
int oracle_direct_f64_at(const float* x, const float* w, const long long* idx, long long n_idx,
                         double* out, int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = oracle_out_size(H, R, s, P), OW = oracle_out_size(W, S, s, P);
    const long long total = (long long)N * K * OH * OW;
    for (long long i = 0; i < n_idx; ++i)
        if (idx[i] < 0 || idx[i] >= total) return 1;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < n_idx; ++i) {
        long long f = idx[i];
        int ow = (int)(f % OW); f /= OW;
        int oh = (int)(f % OH); f /= OH;
        int k = (int)(f % K);
        int n = (int)(f / K);
        out[i] = direct_point(x, w, C, H, W, R, S, s, P, n, k, oh, ow);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Winograd F(2,l) matrices, l = 1, 2, 3                                      */
/* ------------------------------------------------------------------------- */
/*
 * F(2,3): B^T, G, A^T exactly as printed in Sec. 3.2 (the F(2,3) display).
 * F(2,2) and the one-tap case are named by the paper (Sec. 4.1: "apply F(2,2) or
 * F(2,3)") but not printed.  Reading taken here, fixed by Table 3's counts (a
 * 2-tap piece costs 3 multiplications, a 1-tap piece costs 2):
 *   F(2,2): m1=(d0-d1)g0, m2=d1(g0+g1), m3=(d2-d1)g1; y0=m1+m2, y1=m2+m3
 *   F(2,1): m1=d0 g0, m2=d1 g0 (no transform at all)
 * A second F(2,2) with three multiplications is kept beside it (slot 0 of the tables,
 * chosen with oracle_set_f22_form(1)): the one that evaluates at the points 0, 1, -1 --
 * the printed F(2,3) of Sec. 3.2 without its point at infinity, i.e. a 3-tap piece whose
 * third tap is zero, fourth product dropped because it vanishes:
 *   m1=(d0-d2)g0, m2=(d1+d2)(g0+g1)/2, m3=(d2-d1)(g0-g1)/2; y0=m1+m2+m3, y1=m2-m3
 * The paper fixes neither; both are exact, both cost what Table 3 counts.
 * Stored in 4x4 / 4x3 / 2x4 arrays, upper-left corner used: tile length l+1.
 */
static int f22_form_ = 0;
#define LIDX(l) (((l) == 2 && f22_form_) ? 0 : (l))
int oracle_set_f22_form(int form)
{
    if (form != 0 && form != 1) return 1;
    f22_form_ = form;
    return 0;
}
static const double BT_[4][4][4] = {
    /* l=2, points 0,1,-1 */ {{1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 0, 0, 0}},
    /* l=1 */ {{1, 0, 0, 0}, {0, 1, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}},
    /* l=2 */ {{1, -1, 0, 0}, {0, 1, 0, 0}, {0, -1, 1, 0}, {0, 0, 0, 0}},
    /* l=3 */ {{1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 1, 0, -1}},
};
static const double G_[4][4][3] = {
    /* l=2, points 0,1,-1 */ {{1, 0, 0}, {0.5, 0.5, 0}, {0.5, -0.5, 0}, {0, 0, 0}},
    /* l=1 */ {{1, 0, 0}, {1, 0, 0}, {0, 0, 0}, {0, 0, 0}},
    /* l=2 */ {{1, 0, 0}, {1, 1, 0}, {0, 1, 0}, {0, 0, 0}},
    /* l=3 */ {{1, 0, 0}, {0.5, 0.5, 0.5}, {0.5, -0.5, 0.5}, {0, 0, 1}},
};
static const double AT_[4][2][4] = {
    /* l=2, points 0,1,-1 */ {{1, 1, 1, 0}, {0, 1, -1, 0}},
    /* l=1 */ {{1, 0, 0, 0}, {0, 1, 0, 0}},
    /* l=2 */ {{1, 1, 0, 0}, {0, 1, 1, 0}},
    /* l=3 */ {{1, 1, 1, 0}, {0, 1, -1, -1}},
};

/* Copy the matrices of F(2,l) out (row-major BT[(l+1)x(l+1)], G[(l+1)xl], AT[2x(l+1)]). */
int oracle_winograd_matrices(int l, double* BT, double* G, double* AT)
{
    if (l < 1 || l > 3) return 1;
    const int t = l + 1;
    for (int i = 0; i < t; ++i)
        for (int j = 0; j < t; ++j) BT[i * t + j] = BT_[LIDX(l)][i][j];
    for (int i = 0; i < t; ++i)
        for (int j = 0; j < l; ++j) G[i * l + j] = G_[LIDX(l)][i][j];
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < t; ++j) AT[i * t + j] = AT_[LIDX(l)][i][j];
    return 0;
}

/* 1-D F(2,l): Y = A^T [ (G g) .* (B^T d) ]   (Sec. 3.1, the 1-D formula) */
int oracle_winograd_1d(int l, const double* g, const double* d, double* y2)
{
    if (l < 1 || l > 3) return 1;
    const int t = l + 1;
    double u[4], v[4];
    for (int i = 0; i < t; ++i) {
        u[i] = 0.0;
        for (int j = 0; j < l; ++j) u[i] += G_[LIDX(l)][i][j] * g[j];
        v[i] = 0.0;
        for (int j = 0; j < t; ++j) v[i] += BT_[LIDX(l)][i][j] * d[j];
    }
    for (int o = 0; o < 2; ++o) {
        y2[o] = 0.0;
        for (int i = 0; i < t; ++i) y2[o] += AT_[LIDX(l)][o][i] * (u[i] * v[i]);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* O2 step 1: splitting of the kernel                                         */
/* ------------------------------------------------------------------------- */
/*
 * A 1-D piece (p, j, l): phase p (taps whose index is p mod s, Sec. 4.1 eq. 12),
 * offset j inside that phase's tap list, length l in {1,2,3} (Sec. 4.1 eq. 8: the
 * list is cut into threes from the low end, the remainder last; number of cuts is
 * ceil(n_p/3), n_p = ceil((r-p)/s) taps in phase p).  Its taps are g[s*(j+q)+p],
 * q<l.  Only phases that hold a tap exist (p < min(s, r)).
 */
typedef struct { int p, j, l; } oracle_piece;

int oracle_split_1d(int r, int s, oracle_piece* out, int max_out)
{
    int n = 0;
    for (int p = 0; p < s && p < r; ++p) {
        int n_p = (r - p + s - 1) / s;
        for (int j = 0; j < n_p; j += 3) {
            if (n >= max_out) return -1;
            out[n].p = p;
            out[n].j = j;
            out[n].l = (n_p - j < 3) ? (n_p - j) : 3;
            ++n;
        }
    }
    return n;
}

/* A part (sub-kernel) = one piece per dimension ("nest the 1-D methods"). */
typedef struct { int ph, jh, lh, pw, jw, lw; } oracle_part;

#define ORACLE_MAX_PIECES 64

/* parts[] <- cartesian product of the two 1-D splits; returns the count or -1. */
int oracle_split_2d(int R, int S, int s, oracle_part* parts, int max_parts)
{
    oracle_piece hp[ORACLE_MAX_PIECES], wp[ORACLE_MAX_PIECES];
    int nh = oracle_split_1d(R, s, hp, ORACLE_MAX_PIECES);
    int nw = oracle_split_1d(S, s, wp, ORACLE_MAX_PIECES);
    if (nh < 0 || nw < 0 || nh * nw > max_parts) return -1;
    int n = 0;
    for (int a = 0; a < nh; ++a)
        for (int b = 0; b < nw; ++b) {
            parts[n].ph = hp[a].p; parts[n].jh = hp[a].j; parts[n].lh = hp[a].l;
            parts[n].pw = wp[b].p; parts[n].jw = wp[b].j; parts[n].lw = wp[b].l;
            ++n;
        }
    return n;
}

/* Multiplications per 2x2 output tile per (k,c) pair: each part of size lh x lw
 * costs (lh+1)(lw+1) (the counting model behind Table 3). */
long long oracle_mults_per_tile(int R, int S, int s)
{
    oracle_part parts[ORACLE_MAX_PIECES * ORACLE_MAX_PIECES];
    int n = oracle_split_2d(R, S, s, parts, ORACLE_MAX_PIECES * ORACLE_MAX_PIECES);
    if (n < 0) return -1;
    long long m = 0;
    for (int i = 0; i < n; ++i) m += (long long)(parts[i].lh + 1) * (parts[i].lw + 1);
    return m;
}

/* ------------------------------------------------------------------------- */
/* O2 steps 1-2 per part: input slicing + transformation                      */
/* ------------------------------------------------------------------------- */

/* U[K][C][lh+1][lw+1] <- G_lh g G_lw^T,  g[a][b] = w[k][c][s(jh+a)+ph][s(jw+b)+pw] */
int oracle_part_filter_transform(const float* w, int K, int C, int R, int S, int s,
                                 const oracle_part* pt, double* U)
{
    const int lh = pt->lh, lw = pt->lw, th = lh + 1, tw = lw + 1;
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c) {
            double g[3][3], Gg[4][3];
            for (int a = 0; a < lh; ++a)
                for (int b = 0; b < lw; ++b) {
                    int r = s * (pt->jh + a) + pt->ph, q = s * (pt->jw + b) + pt->pw;
                    if (r >= R || q >= S) return 1;
                    g[a][b] = (double)w[(((size_t)k * C + c) * R + r) * S + q];
                }
            for (int i = 0; i < th; ++i)
                for (int b = 0; b < lw; ++b) {
                    Gg[i][b] = 0.0;
                    for (int a = 0; a < lh; ++a) Gg[i][b] += G_[LIDX(lh)][i][a] * g[a][b];
                }
            double* u = U + ((size_t)k * C + c) * th * tw;
            for (int i = 0; i < th; ++i)
                for (int j = 0; j < tw; ++j) {
                    double acc = 0.0;
                    for (int b = 0; b < lw; ++b) acc += Gg[i][b] * G_[LIDX(lw)][j][b];
                    u[i * tw + j] = acc;
                }
        }
    return 0;
}

/*
 * V[C][TH][TW][lh+1][lw+1] for image n <- B_lh^T d B_lw,
 *   d[a][b] = xp[s(2ty+jh+a)+ph][s(2tx+jw+b)+pw]   (phase-p taps meet phase-p samples
 *   of the PADDED input; raw index = padded index - P, zero outside the image).
 * Tiles cover 2x2 output blocks: TH = ceil(OH/2), TW = ceil(OW/2).
 */
int oracle_part_input_transform(const float* x, int C, int H, int W, int s, int P,
                                int TH, int TW, int n, const oracle_part* pt, double* V)
{
    const int lh = pt->lh, lw = pt->lw, th = lh + 1, tw = lw + 1;
    for (int c = 0; c < C; ++c)
        for (int ty = 0; ty < TH; ++ty)
            for (int tx = 0; tx < TW; ++tx) {
                double d[4][4], Bd[4][4];
                for (int a = 0; a < th; ++a)
                    for (int b = 0; b < tw; ++b) {
                        int ih = s * (2 * ty + pt->jh + a) + pt->ph - P;
                        int iw = s * (2 * tx + pt->jw + b) + pt->pw - P;
                        d[a][b] = (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                      ? 0.0
                                      : (double)x[(((size_t)n * C + c) * H + ih) * W + iw];
                    }
                for (int i = 0; i < th; ++i)
                    for (int b = 0; b < tw; ++b) {
                        Bd[i][b] = 0.0;
                        for (int a = 0; a < th; ++a) Bd[i][b] += BT_[LIDX(lh)][i][a] * d[a][b];
                    }
                double* v = V + (((size_t)c * TH + ty) * TW + tx) * th * tw;
                for (int i = 0; i < th; ++i)
                    for (int j = 0; j < tw; ++j) {
                        double acc = 0.0;
                        for (int b = 0; b < tw; ++b) acc += Bd[i][b] * BT_[LIDX(lw)][j][b];
                        v[i * tw + j] = acc;
                    }
            }
    return 0;
}

/*
 * The same transform evaluated in binary32: B^T applied down the columns of the patch first, then
 * along the rows, every sum rounded to binary32.  Each row of B^T has at most two entries (+-1), so
 * each of the two passes is ONE addition or subtraction per output and the order inside a pass does
 * not matter.  With 16-bit inputs the result equals the exact one unless a sum spans more than 13
 * binades (binary16) or 16 binades (bfloat16); it is the arithmetic in which the 16-bit paths decide
 * which 16-bit value an element of V becomes (the paper fixes no precision for its FP16 version).
 */
static int part_input_transform_binary32(const float* x, int C, int H, int W, int s, int P,
                                         int TH, int TW, int n, const oracle_part* pt, double* V)
{
    const int lh = pt->lh, lw = pt->lw, th = lh + 1, tw = lw + 1;
    for (int c = 0; c < C; ++c)
        for (int ty = 0; ty < TH; ++ty)
            for (int tx = 0; tx < TW; ++tx) {
                float d[4][4], Bd[4][4];
                for (int a = 0; a < th; ++a)
                    for (int b = 0; b < tw; ++b) {
                        int ih = s * (2 * ty + pt->jh + a) + pt->ph - P;
                        int iw = s * (2 * tx + pt->jw + b) + pt->pw - P;
                        d[a][b] = (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                      ? 0.0f
                                      : x[(((size_t)n * C + c) * H + ih) * W + iw];
                    }
                for (int i = 0; i < th; ++i)
                    for (int b = 0; b < tw; ++b) {
                        float acc = 0.0f;
                        for (int a = 0; a < th; ++a) {
                            const float coef = (float)BT_[LIDX(lh)][i][a];
                            if (coef != 0.0f) acc = acc + coef * d[a][b];
                        }
                        Bd[i][b] = acc;
                    }
                double* v = V + (((size_t)c * TH + ty) * TW + tx) * th * tw;
                for (int i = 0; i < th; ++i)
                    for (int j = 0; j < tw; ++j) {
                        float acc = 0.0f;
                        for (int b = 0; b < tw; ++b) {
                            const float coef = (float)BT_[LIDX(lw)][j][b];
                            if (coef != 0.0f) acc = acc + coef * Bd[i][b];
                        }
                        v[i * tw + j] = (double)acc;
                    }
            }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* O2: the whole method                                                       */
/* ------------------------------------------------------------------------- */
/*
 * The nearest IEEE binary16 value (ties to even; 11 significant bits, exponents -14..15,
 * subnormals in steps of 2^-24, overflow to infinity from 65520 up), returned as a double.
 */
static double round_binary16(double v)
{
    if (v == 0.0 || v != v || isinf(v)) return v;
    const double a = fabs(v);
    if (a >= 65520.0) return v > 0 ? INFINITY : -INFINITY;
    int e;
    (void)frexp(a, &e);            /* a = m * 2^e, 0.5 <= m < 1: a lies in [2^(e-1), 2^e) */
    int lsb = (e - 1) - 10;        /* weight of the last of 11 significant bits */
    if (lsb < -24) lsb = -24;      /* subnormal range */
    const double ulp = ldexp(1.0, lsb);
    return copysign(nearbyint(a / ulp) * ulp, v); /* default rounding mode: ties to even */
}

int oracle_round_binary16(const double* in, double* out, long long n)
{
    for (long long i = 0; i < n; ++i) out[i] = round_binary16(in[i]);
    return 0;
}

/*
 * The nearest bfloat16 value (ties to even): the format of the same reduced-precision setting
 * on hardware whose matrix units take it -- 8 significant bits, the exponent range of binary32
 * (-126..127), subnormals in steps of 2^-133, overflow to infinity from (2 - 2^-8) * 2^127 up
 * (half a step past the largest finite value (2 - 2^-7) * 2^127).  Returned as a double.
 */
static double round_bfloat16(double v)
{
    if (v == 0.0 || v != v || isinf(v)) return v;
    const double a = fabs(v);
    if (a >= (2.0 - ldexp(1.0, -8)) * ldexp(1.0, 127)) return v > 0 ? INFINITY : -INFINITY;
    int e;
    (void)frexp(a, &e);            /* a lies in [2^(e-1), 2^e) */
    int lsb = (e - 1) - 7;         /* weight of the last of 8 significant bits */
    if (lsb < -133) lsb = -133;    /* subnormal range */
    const double ulp = ldexp(1.0, lsb);
    return copysign(nearbyint(a / ulp) * ulp, v); /* default rounding mode: ties to even */
}

int oracle_round_bfloat16(const double* in, double* out, long long n)
{
    for (long long i = 0; i < n; ++i) out[i] = round_bfloat16(in[i]);
    return 0;
}

static int dwm_forward(const float* x, const float* w, double* y,
                       int N, int C, int H, int W, int K, int R, int S, int s, int P, int half_storage)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = oracle_out_size(H, R, s, P), OW = oracle_out_size(W, S, s, P);
    const int TH = (OH + 1) / 2, TW = (OW + 1) / 2;

    /* Splitting (kernel). */
    oracle_part* parts = (oracle_part*)malloc(sizeof(oracle_part) * ORACLE_MAX_PIECES * ORACLE_MAX_PIECES);
    if (!parts) return 2;
    const int n_parts = oracle_split_2d(R, S, s, parts, ORACLE_MAX_PIECES * ORACLE_MAX_PIECES);
    if (n_parts < 0) { free(parts); return 1; }

    memset(y, 0, sizeof(double) * (size_t)N * K * OH * OW);
    double* U = (double*)malloc(sizeof(double) * (size_t)K * C * 16);
    double* V = (double*)malloc(sizeof(double) * (size_t)C * TH * TW * 16);
    if (!U || !V) { free(parts); free(U); free(V); return 2; }

    int rc = 0;
    for (int ip = 0; ip < n_parts && !rc; ++ip) {
        const oracle_part* pt = &parts[ip];
        const int th = pt->lh + 1, tw = pt->lw + 1;
        /* Transformation (kernel side): U = G g G^T. */
        rc = oracle_part_filter_transform(w, K, C, R, S, s, pt, U);
        if (half_storage && !rc)
            for (size_t i = 0; i < (size_t)K * C * th * tw; ++i)
                U[i] = half_storage == 2 ? round_bfloat16(U[i]) : round_binary16(U[i]);
        for (int n = 0; n < N && !rc; ++n) {
            /* Splitting (input side) + Transformation: V = B^T d B. */
            rc = half_storage ? part_input_transform_binary32(x, C, H, W, s, P, TH, TW, n, pt, V)
                              : oracle_part_input_transform(x, C, H, W, s, P, TH, TW, n, pt, V);
            if (rc) break;
            if (half_storage)
                for (size_t i = 0; i < (size_t)C * TH * TW * th * tw; ++i)
                    V[i] = half_storage == 2 ? round_bfloat16(V[i]) : round_binary16(V[i]);
#pragma omp parallel for schedule(static)
            for (int k = 0; k < K; ++k)
                for (int ty = 0; ty < TH; ++ty)
                    for (int tx = 0; tx < TW; ++tx) {
                        /* Calculation: element-wise product, summed over channels. */
                        double M[4][4];
                        for (int i = 0; i < th; ++i)
                            for (int j = 0; j < tw; ++j) M[i][j] = 0.0;
                        for (int c = 0; c < C; ++c) {
                            const double* u = U + ((size_t)k * C + c) * th * tw;
                            const double* v = V + (((size_t)c * TH + ty) * TW + tx) * th * tw;
                            for (int i = 0; i < th; ++i)
                                for (int j = 0; j < tw; ++j) M[i][j] += u[i * tw + j] * v[i * tw + j];
                        }
                        /* Detransformation: A^T M A. */
                        double AM[2][4];
                        for (int a = 0; a < 2; ++a)
                            for (int j = 0; j < tw; ++j) {
                                AM[a][j] = 0.0;
                                for (int i = 0; i < th; ++i) AM[a][j] += AT_[LIDX(pt->lh)][a][i] * M[i][j];
                            }
                        /* Aggregation: add this part's 2x2 block into the output. */
                        for (int a = 0; a < 2; ++a)
                            for (int b = 0; b < 2; ++b) {
                                int oh = 2 * ty + a, ow = 2 * tx + b;
                                if (oh >= OH || ow >= OW) continue;
                                double acc = 0.0;
                                for (int j = 0; j < tw; ++j) acc += AM[a][j] * AT_[LIDX(pt->lw)][b][j];
                                y[(((size_t)n * K + k) * OH + oh) * OW + ow] += acc;
                            }
                    }
        }
    }
    free(parts); free(U); free(V);
    return rc;
}

int oracle_dwm_f64(const float* x, const float* w, double* y,
                   int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    return dwm_forward(x, w, y, N, C, H, W, K, R, S, s, P, 0);
}

/* O2h: x and w must hold binary16 values (checked); see the header for the rounding points. */
int oracle_dwm_half_f64(const float* x, const float* w, double* y,
                        int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return 1;
    for (size_t i = 0; i < (size_t)N * C * H * W; ++i)
        if (round_binary16((double)x[i]) != (double)x[i]) return 3;
    for (size_t i = 0; i < (size_t)K * C * R * S; ++i)
        if (round_binary16((double)w[i]) != (double)w[i]) return 3;
    return dwm_forward(x, w, y, N, C, H, W, K, R, S, s, P, 1);
}

/* O2b: the same with bfloat16 storage -- x and w must hold bfloat16 values (checked); U and V are
 * rounded once to bfloat16, sums in FP64, the result unrounded. */
int oracle_dwm_bf16_f64(const float* x, const float* w, double* y,
                        int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return 1;
    for (size_t i = 0; i < (size_t)N * C * H * W; ++i)
        if (round_bfloat16((double)x[i]) != (double)x[i]) return 3;
    for (size_t i = 0; i < (size_t)K * C * R * S; ++i)
        if (round_bfloat16((double)w[i]) != (double)w[i]) return 3;
    return dwm_forward(x, w, y, N, C, H, W, K, R, S, s, P, 2);
}

/* ------------------------------------------------------------------------- */
/* Gradient with respect to the input                                         */
/* ------------------------------------------------------------------------- */
/*
 * O1': the definition.  With L = sum_{n,k,oh,ow} dy[n,k,oh,ow] * y[n,k,oh,ow] and y the
 * convolution above, dL/dx[n,c,ih,iw] = sum over every (k, r, q, oh, ow) whose window
 * touches that pixel (oh*s + r - P == ih, ow*s + q - P == iw) of dy[n,k,oh,ow] * w[k,c,r,q].
 * The paper's backward pass (Sec. 3.1 eq. 5 for one Winograd unit, Sec. 4.2 eq. 16-17 for
 * the decomposition: dY^(j) = dY for every part, the parts' input gradients are added up)
 * computes exactly this quantity.
 */
int oracle_backward_data_f64(const float* dy, const float* w, double* dx,
                             int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = (H + 2 * P - R) / s + 1, OW = (W + 2 * P - S) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int ih = 0; ih < H; ++ih)
                for (int iw = 0; iw < W; ++iw) {
                    double acc = 0.0;
                    for (int k = 0; k < K; ++k)
                        for (int r = 0; r < R; ++r) {
                            int a = ih + P - r;
                            if (a < 0 || a % s != 0 || a / s >= OH) continue;
                            for (int q = 0; q < S; ++q) {
                                int b = iw + P - q;
                                if (b < 0 || b % s != 0 || b / s >= OW) continue;
                                acc += (double)dy[(((size_t)n * K + k) * OH + a / s) * OW + b / s] *
                                       (double)w[(((size_t)k * C + c) * R + r) * S + q];
                            }
                        }
                    dx[(((size_t)n * C + c) * H + ih) * W + iw] = acc;
                }
    return 0;
}

/* O1' at sampled positions of dx (flat indices into [N][C][H][W]). */
int oracle_backward_data_f64_at(const float* dy, const float* w, const long long* idx, long long n_idx, double* out,
                                int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = (H + 2 * P - R) / s + 1, OW = (W + 2 * P - S) / s + 1;
    const long long total = (long long)N * C * H * W;
    for (long long i = 0; i < n_idx; ++i)
        if (idx[i] < 0 || idx[i] >= total) return 1;
#pragma omp parallel for schedule(dynamic, 64)
    for (long long i = 0; i < n_idx; ++i) {
        long long e = idx[i];
        const int iw = (int)(e % W); e /= W;
        const int ih = (int)(e % H); e /= H;
        const int c = (int)(e % C);
        const int n = (int)(e / C);
        double acc = 0.0;
        for (int k = 0; k < K; ++k)
            for (int r = 0; r < R; ++r) {
                int a = ih + P - r;
                if (a < 0 || a % s != 0 || a / s >= OH) continue;
                for (int q = 0; q < S; ++q) {
                    int b = iw + P - q;
                    if (b < 0 || b % s != 0 || b / s >= OW) continue;
                    acc += (double)dy[(((size_t)n * K + k) * OH + a / s) * OW + b / s] *
                           (double)w[(((size_t)k * C + c) * R + r) * S + q];
                }
            }
        out[i] = acc;
    }
    return 0;
}

/*
 * O2': the paper's backward pass step by step.  For every part (splitting as in the
 * forward pass) and every 2x2 output tile: dM = A dY A^T (the transposed
 * detransformation), dV = sum_k U .* dM (Sec. 3.1 eq. 5: dd = B[(A dY A^T) .* U]B^T, with
 * the sum over filters that the channel-wise forward sum turns into), dd = B dV B^T, and
 * dd is added into the padded input gradient at the positions the part's patch was read
 * from (Sec. 4.2 eq. 17: the parts' gradients are summed).  The padding is cropped last.
 */
int oracle_dwm_backward_data_f64(const float* dy, const float* w, double* dx,
                                 int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = (H + 2 * P - R) / s + 1, OW = (W + 2 * P - S) / s + 1;
    const int TH = (OH + 1) / 2, TW = (OW + 1) / 2;
    /* padded gradient image, large enough for the overhang of the last (partial) tile */
    const int HP = s * (2 * TH + (R + s - 1) / s + 2) + s, WP = s * (2 * TW + (S + s - 1) / s + 2) + s;
    oracle_part* parts = (oracle_part*)malloc(sizeof(oracle_part) * ORACLE_MAX_PIECES * ORACLE_MAX_PIECES);
    if (!parts) return 2;
    const int n_parts = oracle_split_2d(R, S, s, parts, ORACLE_MAX_PIECES * ORACLE_MAX_PIECES);
    if (n_parts < 0) { free(parts); return 1; }
    double* U = (double*)malloc(sizeof(double) * (size_t)K * C * 16);
    double* gp = (double*)malloc(sizeof(double) * (size_t)C * HP * WP);
    if (!U || !gp) { free(parts); free(U); free(gp); return 2; }
    int rc = 0;
    for (int n = 0; n < N && !rc; ++n) {
        memset(gp, 0, sizeof(double) * (size_t)C * HP * WP);
        for (int ip = 0; ip < n_parts && !rc; ++ip) {
            const oracle_part* pt = &parts[ip];
            const int th = pt->lh + 1, tw = pt->lw + 1;
            rc = oracle_part_filter_transform(w, K, C, R, S, s, pt, U);
            if (rc) break;
#pragma omp parallel for schedule(static)
            for (int c = 0; c < C; ++c)
                for (int ty = 0; ty < TH; ++ty)
                    for (int tx = 0; tx < TW; ++tx) {
                        double dV[4][4];
                        for (int i = 0; i < th; ++i)
                            for (int j = 0; j < tw; ++j) dV[i][j] = 0.0;
                        for (int k = 0; k < K; ++k) {
                            /* dM = A dY A^T, dY the tile's 2x2 block (zero past the output) */
                            double g2[2][2], Ag[4][2];
                            for (int a = 0; a < 2; ++a)
                                for (int b = 0; b < 2; ++b) {
                                    int oh = 2 * ty + a, ow = 2 * tx + b;
                                    g2[a][b] = (oh < OH && ow < OW)
                                                   ? (double)dy[(((size_t)n * K + k) * OH + oh) * OW + ow] : 0.0;
                                }
                            for (int i = 0; i < th; ++i)
                                for (int b = 0; b < 2; ++b) {
                                    Ag[i][b] = 0.0;
                                    for (int a = 0; a < 2; ++a) Ag[i][b] += AT_[LIDX(pt->lh)][a][i] * g2[a][b];
                                }
                            const double* u = U + ((size_t)k * C + c) * th * tw;
                            for (int i = 0; i < th; ++i)
                                for (int j = 0; j < tw; ++j) {
                                    double dM = 0.0;
                                    for (int b = 0; b < 2; ++b) dM += Ag[i][b] * AT_[LIDX(pt->lw)][b][j];
                                    dV[i][j] += u[i * tw + j] * dM;
                                }
                        }
                        /* dd = B dV B^T, added where the patch was read */
                        double BdV[4][4];
                        for (int a = 0; a < th; ++a)
                            for (int j = 0; j < tw; ++j) {
                                BdV[a][j] = 0.0;
                                for (int i = 0; i < th; ++i) BdV[a][j] += BT_[LIDX(pt->lh)][i][a] * dV[i][j];
                            }
                        for (int a = 0; a < th; ++a)
                            for (int b = 0; b < tw; ++b) {
                                double acc = 0.0;
                                for (int j = 0; j < tw; ++j) acc += BdV[a][j] * BT_[LIDX(pt->lw)][j][b];
                                int ph = s * (2 * ty + pt->jh + a) + pt->ph, pw = s * (2 * tx + pt->jw + b) + pt->pw;
                                gp[((size_t)c * HP + ph) * WP + pw] += acc;
                            }
                    }
        }
        for (int c = 0; c < C; ++c)
            for (int ih = 0; ih < H; ++ih)
                for (int iw = 0; iw < W; ++iw)
                    dx[(((size_t)n * C + c) * H + ih) * W + iw] = gp[((size_t)c * HP + ih + P) * WP + iw + P];
    }
    free(parts); free(U); free(gp);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Gradient with respect to the filter                                        */
/* ------------------------------------------------------------------------- */
/*
 * O1'': the definition.  y is linear in w, so for L = sum dy * y
 *   dL/dw[k,c,r,q] = sum_{n,oh,ow} dy[n,k,oh,ow] * xp[n,c,oh*s+r,ow*s+q]   (xp = padded x).
 * The paper's backward pass (Sec. 3.1 eq. 5, second formula; Sec. 4.2 eq. 18: every part's
 * kernel gradient is computed from the whole output gradient) computes this quantity.
 */
int oracle_backward_filter_f64(const float* x, const float* dy, double* dw,
                               int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = (H + 2 * P - R) / s + 1, OW = (W + 2 * P - S) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int q = 0; q < S; ++q) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int oh = 0; oh < OH; ++oh) {
                            int ih = oh * s + r - P;
                            if (ih < 0 || ih >= H) continue;
                            for (int ow = 0; ow < OW; ++ow) {
                                int iw = ow * s + q - P;
                                if (iw < 0 || iw >= W) continue;
                                acc += (double)dy[(((size_t)n * K + k) * OH + oh) * OW + ow] *
                                       (double)x[(((size_t)n * C + c) * H + ih) * W + iw];
                            }
                        }
                    dw[(((size_t)k * C + c) * R + r) * S + q] = acc;
                }
    return 0;
}

/*
 * O2'': the paper's formula part by part: dg = G^T [ sum over tiles and images of
 * (A dY A^T) .* V ] G (Sec. 3.1 eq. 5), V = B^T d B the part's transformed input patch;
 * a part's dg lands on the taps the part was cut from (Sec. 4.2 eq. 18).
 */
int oracle_dwm_backward_filter_f64(const float* x, const float* dy, double* dw,
                                   int N, int C, int H, int W, int K, int R, int S, int s, int P)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 || s < 1 || P < 0) return 1;
    if (H + 2 * P < R || W + 2 * P < S) return 1;
    const int OH = (H + 2 * P - R) / s + 1, OW = (W + 2 * P - S) / s + 1;
    const int TH = (OH + 1) / 2, TW = (OW + 1) / 2;
    oracle_part* parts = (oracle_part*)malloc(sizeof(oracle_part) * ORACLE_MAX_PIECES * ORACLE_MAX_PIECES);
    if (!parts) return 2;
    const int n_parts = oracle_split_2d(R, S, s, parts, ORACLE_MAX_PIECES * ORACLE_MAX_PIECES);
    if (n_parts < 0) { free(parts); return 1; }
    double* V = (double*)malloc(sizeof(double) * (size_t)C * TH * TW * 16);
    double* dU = (double*)malloc(sizeof(double) * (size_t)K * C * 16);
    if (!V || !dU) { free(parts); free(V); free(dU); return 2; }
    memset(dw, 0, sizeof(double) * (size_t)K * C * R * S);
    int rc = 0;
    for (int ip = 0; ip < n_parts && !rc; ++ip) {
        const oracle_part* pt = &parts[ip];
        const int lh = pt->lh, lw = pt->lw, th = lh + 1, tw = lw + 1;
        memset(dU, 0, sizeof(double) * (size_t)K * C * 16);
        for (int n = 0; n < N && !rc; ++n) {
            rc = oracle_part_input_transform(x, C, H, W, s, P, TH, TW, n, pt, V);
            if (rc) break;
#pragma omp parallel for schedule(static)
            for (int k = 0; k < K; ++k)
                for (int ty = 0; ty < TH; ++ty)
                    for (int tx = 0; tx < TW; ++tx) {
                        double g2[2][2], Ag[4][2], dM[4][4];
                        for (int a = 0; a < 2; ++a)
                            for (int b = 0; b < 2; ++b) {
                                int oh = 2 * ty + a, ow = 2 * tx + b;
                                g2[a][b] = (oh < OH && ow < OW)
                                               ? (double)dy[(((size_t)n * K + k) * OH + oh) * OW + ow] : 0.0;
                            }
                        for (int i = 0; i < th; ++i)
                            for (int b = 0; b < 2; ++b) {
                                Ag[i][b] = 0.0;
                                for (int a = 0; a < 2; ++a) Ag[i][b] += AT_[LIDX(lh)][a][i] * g2[a][b];
                            }
                        for (int i = 0; i < th; ++i)
                            for (int j = 0; j < tw; ++j) {
                                dM[i][j] = 0.0;
                                for (int b = 0; b < 2; ++b) dM[i][j] += Ag[i][b] * AT_[LIDX(lw)][b][j];
                            }
                        for (int c = 0; c < C; ++c) {
                            const double* v = V + (((size_t)c * TH + ty) * TW + tx) * th * tw;
                            double* du = dU + ((size_t)k * C + c) * 16;
                            for (int i = 0; i < th; ++i)
                                for (int j = 0; j < tw; ++j) du[i * 4 + j] += dM[i][j] * v[i * tw + j];
                        }
                    }
        }
        /* dg = G^T dU G onto the part's taps */
        for (int k = 0; k < K && !rc; ++k)
            for (int c = 0; c < C; ++c) {
                const double* du = dU + ((size_t)k * C + c) * 16;
                for (int a = 0; a < lh; ++a)
                    for (int b = 0; b < lw; ++b) {
                        double acc = 0.0;
                        for (int i = 0; i < th; ++i)
                            for (int j = 0; j < tw; ++j)
                                acc += G_[LIDX(lh)][i][a] * du[i * 4 + j] * G_[LIDX(lw)][j][b];
                        int r = s * (pt->jh + a) + pt->ph, q = s * (pt->jw + b) + pt->pw;
                        dw[(((size_t)k * C + c) * R + r) * S + q] += acc;
                    }
            }
    }
    free(parts); free(V); free(dU);
    return rc;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
