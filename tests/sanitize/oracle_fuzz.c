/* Host-only fuzz of the oracle's C code, built with -fsanitize=address,undefined by
 * tests/test_sanitize.py: random tiny shapes through every entry point, outputs in exactly sized
 * heap buffers so that any access past them is caught; the FP64 DWM must equal the definitions. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/dwm_oracle.c"

static uint64_t g_state = 0x243F6A8885A308D3ull;
static uint32_t rnd(void)
{
    g_state ^= g_state << 13;
    g_state ^= g_state >> 7;
    g_state ^= g_state << 17;
    return (uint32_t)(g_state >> 32);
}
static int pick(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }
static float unit(void) { return (float)((double)rnd() / 4294967296.0 * 2.0 - 1.0); }

#define CHECK(c)                                                                        \
    do {                                                                                \
        if (!(c)) {                                                                     \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c);       \
            exit(2);                                                                    \
        }                                                                               \
    } while (0)

static double maxdiff(const double* a, const double* b, size_t n, double* scale)
{
    double m = 0, s = 0;
    for (size_t i = 0; i < n; ++i) {
        if (fabs(a[i] - b[i]) > m) m = fabs(a[i] - b[i]);
        if (fabs(b[i]) > s) s = fabs(b[i]);
    }
    *scale = s > 0 ? s : 1;
    return m;
}

int main(int argc, char** argv)
{
    const int iters = argc > 1 ? atoi(argv[1]) : 300;
    for (int it = 0; it < iters; ++it) {
        const int R = pick(1, 11), S = pick(1, 11), s = pick(1, 4), P = pick(0, 5);
        const int H = pick(1, 14), W = pick(1, 14), C = pick(1, 3), K = pick(1, 3), N = pick(1, 2);
        oracle_set_f22_form(it & 1);
        if (H + 2 * P < R || W + 2 * P < S) {
            double y;
            float x = 0, w = 0;
            CHECK(oracle_direct_f64(&x, &w, &y, N, C, H, W, K, R, S, s, P) != 0);
            continue;
        }
        const int OH = oracle_out_size(H, R, s, P), OW = oracle_out_size(W, S, s, P);
        const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * C * R * S, ny = (size_t)N * K * OH * OW;
        float* x = malloc(nx * sizeof(float));
        float* w = malloc(nw * sizeof(float));
        float* dy = malloc(ny * sizeof(float));
        double* y1 = malloc(ny * sizeof(double));
        double* y2 = malloc(ny * sizeof(double));
        double* dx1 = malloc(nx * sizeof(double));
        double* dx2 = malloc(nx * sizeof(double));
        double* dw1 = malloc(nw * sizeof(double));
        double* dw2 = malloc(nw * sizeof(double));
        for (size_t i = 0; i < nx; ++i) x[i] = unit();
        for (size_t i = 0; i < nw; ++i) w[i] = unit();
        for (size_t i = 0; i < ny; ++i) dy[i] = unit();
        double sc;
        CHECK(oracle_direct_f64(x, w, y1, N, C, H, W, K, R, S, s, P) == 0);
        CHECK(oracle_dwm_f64(x, w, y2, N, C, H, W, K, R, S, s, P) == 0);
        CHECK(maxdiff(y2, y1, ny, &sc) <= 1e-12 * sc);
        /* sampled form: every index, and one past the end is refused */
        long long* idx = malloc((ny + 1) * sizeof(long long));
        for (size_t i = 0; i <= ny; ++i) idx[i] = (long long)i;
        CHECK(oracle_direct_f64_at(x, w, idx, (long long)ny, y2, N, C, H, W, K, R, S, s, P) == 0);
        CHECK(maxdiff(y2, y1, ny, &sc) == 0);
        CHECK(oracle_direct_f64_at(x, w, idx, (long long)ny + 1, y2, N, C, H, W, K, R, S, s, P) != 0);
        CHECK(oracle_backward_data_f64(dy, w, dx1, N, C, H, W, K, R, S, s, P) == 0);
        CHECK(oracle_dwm_backward_data_f64(dy, w, dx2, N, C, H, W, K, R, S, s, P) == 0);
        CHECK(maxdiff(dx2, dx1, nx, &sc) <= 1e-12 * sc);
        CHECK(oracle_backward_filter_f64(x, dy, dw1, N, C, H, W, K, R, S, s, P) == 0);
        CHECK(oracle_dwm_backward_filter_f64(x, dy, dw2, N, C, H, W, K, R, S, s, P) == 0);
        CHECK(maxdiff(dw2, dw1, nw, &sc) <= 1e-12 * sc);
        /* the splitting and the per-part transforms, outputs sized exactly */
        oracle_part parts[256];
        const int np = oracle_split_2d(R, S, s, parts, 256);
        CHECK(np > 0 && np <= 256);
        CHECK(oracle_split_2d(R, S, s, parts, np - 1) < 0);
        for (int i = 0; i < np; ++i) {
            const int th = parts[i].lh + 1, tw = parts[i].lw + 1;
            double* U = malloc((size_t)K * C * th * tw * sizeof(double));
            CHECK(oracle_part_filter_transform(w, K, C, R, S, s, &parts[i], U) == 0);
            free(U);
            const int TH = (OH + 1) / 2, TW = (OW + 1) / 2;
            double* V = malloc((size_t)C * TH * TW * th * tw * sizeof(double));
            CHECK(oracle_part_input_transform(x, C, H, W, s, P, TH, TW, N - 1, &parts[i], V) == 0);
            free(V);
        }
        free(idx); free(x); free(w); free(dy); free(y1); free(y2); free(dx1); free(dx2); free(dw1); free(dw2);
    }
    /* the rounding to binary16 over special values */
    double in[] = {0.0, -0.0, 1.0, 65504.0, 65519.99, 65520.0, 1e30, -1e30, 5.960464477539063e-08, 2.9e-8, 3.0e-8, 1e-300};
    double out[sizeof(in) / sizeof(in[0])];
    CHECK(oracle_round_binary16(in, out, (long long)(sizeof(in) / sizeof(in[0]))) == 0);
    CHECK(out[3] == 65504.0 && out[4] == 65504.0 && isinf(out[5]) && out[11] == 0.0);
    printf("oracle fuzz: %d shapes\n", iters);
    return 0;
}
