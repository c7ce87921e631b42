/*
 * CPU oracle, part 1 of 2: the convolution and pooling definitions in double precision.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain-definition checker for the
 * HIP library; it shares no code with it and the product path never calls it.
 *
 * The residual function F of a block (Sec. 2.1, the layer-serial training task, and
 * Sec. 4.1, the decoupled feature flow) is built from convolutions; its Jacobian
 * products dF/dX and dF/dW in the discrete adjoint and the weight update of Sec. 4.1
 * are the data-gradient and weight-gradient below.  Each routine is the textbook
 * definition written as nested loops over NHWC activations [N,H,W,C] and KRSC
 * filters [Cout,R,S,Cin]; OpenMP only splits an outer loop whose iterations write
 * disjoint outputs, so no reduction is reordered between threads.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int lpref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Y[n,ho,wo,co] = sum_{r,s,ci} X[n, ho*stride-pad+r, wo*stride-pad+s, ci] * W[co,r,s,ci]  */
void lpref_conv_fwd(const double* x, const double* w, double* y,
                    int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad) {
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
    const long rows = (long)N * Ho;
#pragma omp parallel for schedule(static)
    for (long nh = 0; nh < rows; ++nh) {
        const int n = (int)(nh / Ho), ho = (int)(nh % Ho);
        for (int wo = 0; wo < Wo; ++wo)
            for (int co = 0; co < Cout; ++co) {
                double acc = 0.0;
                for (int r = 0; r < R; ++r) {
                    const int hi = ho * stride - pad + r;
                    if (hi < 0 || hi >= H) continue;
                    for (int s = 0; s < S; ++s) {
                        const int wi = wo * stride - pad + s;
                        if (wi < 0 || wi >= W) continue;
                        const double* xp = x + (((size_t)n * H + hi) * W + wi) * Cin;
                        const double* wp = w + (((size_t)co * R + r) * S + s) * Cin;
                        for (int ci = 0; ci < Cin; ++ci) acc += xp[ci] * wp[ci];
                    }
                }
                y[(((size_t)n * Ho + ho) * Wo + wo) * Cout + co] = acc;
            }
    }
}

/* One output element of the forward convolution (for sampled checks at large sizes). */
double lpref_conv_fwd_at(const double* x, const double* w,
                         int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad,
                         int n, int ho, int wo, int co) {
    (void)N; (void)Cout;
    double acc = 0.0;
    for (int r = 0; r < R; ++r) {
        const int hi = ho * stride - pad + r;
        if (hi < 0 || hi >= H) continue;
        for (int s = 0; s < S; ++s) {
            const int wi = wo * stride - pad + s;
            if (wi < 0 || wi >= W) continue;
            const double* xp = x + (((size_t)n * H + hi) * W + wi) * Cin;
            const double* wp = w + (((size_t)co * R + r) * S + s) * Cin;
            for (int ci = 0; ci < Cin; ++ci) acc += xp[ci] * wp[ci];
        }
    }
    return acc;
}

/* dX = (dY/dX)^T dY: every forward product x*w contributes w*dy to dX at the same x index. */
void lpref_conv_dgrad(const double* dy, const double* w, double* dx,
                      int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad) {
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
    memset(dx, 0, sizeof(double) * (size_t)N * H * W * Cin);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int co = 0; co < Cout; ++co) {
                    const double g = dy[(((size_t)n * Ho + ho) * Wo + wo) * Cout + co];
                    for (int r = 0; r < R; ++r) {
                        const int hi = ho * stride - pad + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int wi = wo * stride - pad + s;
                            if (wi < 0 || wi >= W) continue;
                            double* dxp = dx + (((size_t)n * H + hi) * W + wi) * Cin;
                            const double* wp = w + (((size_t)co * R + r) * S + s) * Cin;
                            for (int ci = 0; ci < Cin; ++ci) dxp[ci] += g * wp[ci];
                        }
                    }
                }
}

/* dW[co,r,s,ci] = sum_{n,ho,wo} dY[n,ho,wo,co] * X[n, ho*stride-pad+r, wo*stride-pad+s, ci] */
void lpref_conv_wgrad(const double* x, const double* dy, double* dw,
                      int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad) {
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
    memset(dw, 0, sizeof(double) * (size_t)Cout * R * S * Cin);
#pragma omp parallel for schedule(static)
    for (int co = 0; co < Cout; ++co)
        for (int n = 0; n < N; ++n)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    const double g = dy[(((size_t)n * Ho + ho) * Wo + wo) * Cout + co];
                    for (int r = 0; r < R; ++r) {
                        const int hi = ho * stride - pad + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int wi = wo * stride - pad + s;
                            if (wi < 0 || wi >= W) continue;
                            const double* xp = x + (((size_t)n * H + hi) * W + wi) * Cin;
                            double* dwp = dw + (((size_t)co * R + r) * S + s) * Cin;
                            for (int ci = 0; ci < Cin; ++ci) dwp[ci] += g * xp[ci];
                        }
                    }
                }
}

/*
 * Canonical im2col address: element (m, q) of the implicit GEMM operand of a forward
 * convolution, m = (n*Ho+ho)*Wo+wo, q = (r*S+s)*Cin+ci.  Returns the flat NHWC offset of the
 * activation it reads, or -1 when the tap falls into the zero padding.
 */
int64_t lpref_im2col_index(int64_t m, int64_t q, int H, int W, int Cin, int R, int S, int stride, int pad) {
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
    const int64_t n = m / ((int64_t)Ho * Wo);
    const int ho = (int)((m / Wo) % Ho), wo = (int)(m % Wo);
    const int r = (int)(q / ((int64_t)S * Cin)), s = (int)((q / Cin) % S), ci = (int)(q % Cin);
    const int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
    if (hi < 0 || hi >= H || wi < 0 || wi >= W) return -1;
    return ((n * H + hi) * W + wi) * Cin + ci;
}

/* Max pooling; idx holds the flat input offset of the first maximum in row-major window order. */
void lpref_maxpool_fwd(const double* x, double* y, int64_t* idx,
                       int N, int H, int W, int C, int R, int stride, int pad) {
    const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - R) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int c = 0; c < C; ++c) {
                    double best = 0.0; int64_t bi = -1;
                    for (int r = 0; r < R; ++r) {
                        const int hi = ho * stride - pad + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int s = 0; s < R; ++s) {
                            const int wi = wo * stride - pad + s;
                            if (wi < 0 || wi >= W) continue;
                            const int64_t o = (((int64_t)n * H + hi) * W + wi) * C + c;
                            if (bi < 0 || x[o] > best) { best = x[o]; bi = o; }
                        }
                    }
                    const size_t oo = (((size_t)n * Ho + ho) * Wo + wo) * C + c;
                    y[oo] = best; idx[oo] = bi;
                }
}

void lpref_maxpool_bwd(const double* dy, const int64_t* idx, double* dx, int64_t n_out, int64_t n_in) {
    memset(dx, 0, sizeof(double) * (size_t)n_in);
    for (int64_t i = 0; i < n_out; ++i) dx[idx[i]] += dy[i];
}
