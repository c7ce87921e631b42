/*
 * Self-check of the oracle's C part, meant to be built with -fsanitize=address,undefined (oracle/build.py,
 * build_selfcheck): it drives every routine of lpref.c over small ragged shapes (strides 1 and 2, filters 1, 3 and 7
 * wide, paddings 0..3, odd image sizes) and checks results that do not come from the routines themselves:
 *   - lpref_conv_fwd against a gather through lpref_im2col_index, and lpref_conv_fwd_at against both;
 *   - the adjoint identities  <conv(x,w), g> = <x, dgrad(g,w)> = <w, wgrad(x,g)>  (bilinearity of the convolution);
 *   - max pooling: every output is the maximum of its window, the recorded index points at it, and the backward
 *     pass scatters each gradient to exactly that index.
 * TEST INFRASTRUCTURE ONLY, like lpref.c.  Exit status 0: everything held and the sanitizers saw nothing.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "lpref.c"

static uint64_t rng_state = 0x2112053872112053ull;
static double rnd(void) {                       /* SplitMix64 -> uniform in (-1, 1) */
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (double)(z >> 11) / 4503599627370496.0 - 1.0;
}
static double* vec(size_t n) {
    double* p = (double*)malloc((n ? n : 1) * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
static double dot(const double* a, const double* b, size_t n) {
    double s = 0;
    for (size_t i = 0; i < n; ++i) s += a[i] * b[i];
    return s;
}
static int fails = 0;
static void expect(int ok, const char* what, int N, int H, int W, int Cin, int Cout, int R, int stride, int pad) {
    if (!ok) {
        ++fails;
        fprintf(stderr, "FAILED %s: N=%d H=%d W=%d Cin=%d Cout=%d R=%d stride=%d pad=%d\n", what, N, H, W, Cin, Cout, R, stride, pad);
    }
}

static void check_conv(int N, int H, int W, int Cin, int Cout, int R, int stride, int pad) {
    const int S = R;
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
    const size_t nx = (size_t)N * H * W * Cin, nw = (size_t)Cout * R * S * Cin, ny = (size_t)N * Ho * Wo * Cout;
    double *x = vec(nx), *w = vec(nw), *g = vec(ny), *y = vec(ny), *dx = vec(nx), *dw = vec(nw);
    lpref_conv_fwd(x, w, y, N, H, W, Cin, Cout, R, S, stride, pad);
    /* forward against the index function */
    double worst = 0;
    for (int64_t m = 0; m < (int64_t)N * Ho * Wo; ++m)
        for (int co = 0; co < Cout; ++co) {
            double s = 0;
            for (int64_t q = 0; q < (int64_t)R * S * Cin; ++q) {
                const int64_t off = lpref_im2col_index(m, q, H, W, Cin, R, S, stride, pad);
                if (off >= 0) s += x[off] * w[(size_t)co * R * S * Cin + q];
            }
            const double d = fabs(s - y[m * Cout + co]);
            if (d > worst) worst = d;
            const int n = (int)(m / ((int64_t)Ho * Wo)), ho = (int)((m / Wo) % Ho), wo = (int)(m % Wo);
            const double at = lpref_conv_fwd_at(x, w, N, H, W, Cin, Cout, R, S, stride, pad, n, ho, wo, co);
            if (fabs(at - y[m * Cout + co]) > worst) worst = fabs(at - y[m * Cout + co]);
        }
    expect(worst < 1e-12, "conv_fwd vs im2col gather", N, H, W, Cin, Cout, R, stride, pad);
    /* adjoint identities */
    lpref_conv_dgrad(g, w, dx, N, H, W, Cin, Cout, R, S, stride, pad);
    lpref_conv_wgrad(x, g, dw, N, H, W, Cin, Cout, R, S, stride, pad);
    const double a = dot(y, g, ny), b = dot(x, dx, nx), c = dot(w, dw, nw);
    const double scale = fabs(a) + 1.0;
    expect(fabs(a - b) < 1e-10 * scale && fabs(a - c) < 1e-10 * scale, "adjoint identities", N, H, W, Cin, Cout, R, stride, pad);
    free(x); free(w); free(g); free(y); free(dx); free(dw);
}

static void check_pool(int N, int H, int W, int C, int R, int stride, int pad) {
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - R) / stride + 1;
    const size_t nx = (size_t)N * H * W * C, ny = (size_t)N * Ho * Wo * C;
    double *x = vec(nx), *y = vec(ny), *g = vec(ny), *dx = vec(nx);
    int64_t* idx = (int64_t*)malloc((ny ? ny : 1) * sizeof(int64_t));
    lpref_maxpool_fwd(x, y, idx, N, H, W, C, R, stride, pad);
    int ok = 1;
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int c = 0; c < C; ++c) {
                    const size_t o = (((size_t)n * Ho + ho) * Wo + wo) * C + c;
                    double best = -INFINITY;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < R; ++s) {
                            const int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
                            if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                            const double v = x[(((size_t)n * H + hi) * W + wi) * C + c];
                            if (v > best) best = v;
                        }
                    ok = ok && y[o] == best && idx[o] >= 0 && (size_t)idx[o] < nx && x[idx[o]] == best;
                }
    lpref_maxpool_bwd(g, idx, dx, (int64_t)ny, (int64_t)nx);
    double* want = (double*)calloc(nx ? nx : 1, sizeof(double));
    for (size_t o = 0; o < ny; ++o) want[idx[o]] += g[o];
    for (size_t i = 0; i < nx; ++i) ok = ok && fabs(want[i] - dx[i]) < 1e-12;
    expect(ok, "max pooling", N, H, W, C, C, R, stride, pad);
    free(x); free(y); free(g); free(dx); free(idx); free(want);
}

int main(void) {
    static const int cases[][8] = {      /* N, H, W, Cin, Cout, R, stride, pad */
        {2, 5, 7, 3, 4, 3, 1, 1}, {1, 6, 6, 2, 3, 3, 2, 1}, {2, 9, 7, 3, 2, 7, 2, 3}, {3, 4, 5, 5, 6, 1, 1, 0},
        {1, 8, 6, 4, 4, 1, 2, 0}, {2, 3, 3, 1, 1, 3, 1, 0}, {1, 1, 1, 2, 3, 3, 1, 1}, {2, 7, 5, 2, 2, 3, 2, 0},
        {1, 10, 4, 3, 5, 3, 1, 2}, {2, 4, 4, 8, 8, 3, 1, 1}};
    for (size_t i = 0; i < sizeof(cases) / sizeof(cases[0]); ++i)
        check_conv(cases[i][0], cases[i][1], cases[i][2], cases[i][3], cases[i][4], cases[i][5], cases[i][6], cases[i][7]);
    check_pool(2, 8, 8, 3, 3, 2, 1);
    check_pool(1, 7, 9, 2, 3, 2, 1);
    check_pool(2, 5, 5, 4, 2, 2, 0);
    printf("lpref self-check: %d failure(s), %d thread(s)\n", fails, lpref_num_threads());
    return fails ? 1 : 0;
}
