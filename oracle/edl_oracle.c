/*
 * CPU oracle for one worker's synchronous-SGD iteration (paper section 2.1:
 * the mini-batch SGD update and the synchronous data-parallel scheme).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain nested loops, IEEE double everywhere, no
 * blocking, no fusion.  Shares no code with the HIP path.  Only tests, the
 * smoke check and the bench's cpu_baseline leg may call this.
 *
 * Layouts: activations are [N][H][W][C] (channels innermost); convolution
 * weights are [K][R][S][C] (output channel, kernel row, kernel column, input
 * channel).  A convolution is a cross-correlation with zero padding:
 *
 *   y[n,ho,wo,k] = b[k] + sum_{r,s,c} x[n, ho*st - pad + r, wo*st - pad + s, c] * w[k,r,s,c]
 *
 * The three routines below are that definition and its two partial
 * derivatives written out.  OpenMP only splits the outermost independent
 * loop; every output element is still accumulated by exactly one thread in
 * the loop order shown.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

static inline int out_extent(int in, int k, int stride, int pad) {
    return (in + 2 * pad - k) / stride + 1;
}

/* y = conv(x, w) + b.  b may be NULL. */
void oracle_conv2d_forward(const double* x, const double* w, const double* b, double* y,
                           int N, int H, int W, int C, int K, int R, int S, int stride, int pad)
{
    const int Ho = out_extent(H, R, stride, pad), Wo = out_extent(W, S, stride, pad);
    #pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
    for (int wo = 0; wo < Wo; ++wo) {
        double* yrow = y + (((size_t)n * Ho + ho) * Wo + wo) * K;
        for (int k = 0; k < K; ++k) {
            double acc = b ? b[k] : 0.0;
            for (int r = 0; r < R; ++r) {
                const int h = ho * stride - pad + r;
                if (h < 0 || h >= H) continue;
                for (int s = 0; s < S; ++s) {
                    const int wi = wo * stride - pad + s;
                    if (wi < 0 || wi >= W) continue;
                    const double* xp = x + (((size_t)n * H + h) * W + wi) * C;
                    const double* wp = w + (((size_t)k * R + r) * S + s) * C;
                    double part = 0.0;
                    #pragma omp simd reduction(+:part)
                    for (int c = 0; c < C; ++c) part += xp[c] * wp[c];
                    acc += part;
                }
            }
            yrow[k] = acc;
        }
    }
}

/* dx[n,h,w,c] = sum_{k,r,s} dy[n,ho,wo,k] * w[k,r,s,c] over all (ho,wo,r,s) with
 * ho*st - pad + r == h and wo*st - pad + s == w.  dx is overwritten. */
void oracle_conv2d_backward_input(const double* dy, const double* w, double* dx,
                                  int N, int H, int W, int C, int K, int R, int S, int stride, int pad)
{
    const int Ho = out_extent(H, R, stride, pad), Wo = out_extent(W, S, stride, pad);
    #pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
    for (int h = 0; h < H; ++h)
    for (int wi = 0; wi < W; ++wi) {
        double* dxp = dx + (((size_t)n * H + h) * W + wi) * C;
        for (int c = 0; c < C; ++c) dxp[c] = 0.0;
        for (int r = 0; r < R; ++r) {
            const int hn = h + pad - r;
            if (hn < 0 || hn % stride != 0) continue;
            const int ho = hn / stride;
            if (ho >= Ho) continue;
            for (int s = 0; s < S; ++s) {
                const int wn = wi + pad - s;
                if (wn < 0 || wn % stride != 0) continue;
                const int wo = wn / stride;
                if (wo >= Wo) continue;
                const double* dyp = dy + (((size_t)n * Ho + ho) * Wo + wo) * K;
                for (int k = 0; k < K; ++k) {
                    const double g = dyp[k];
                    const double* wp = w + (((size_t)k * R + r) * S + s) * C;
                    for (int c = 0; c < C; ++c) dxp[c] += g * wp[c];
                }
            }
        }
    }
}

/* dw[k,r,s,c] = sum_{n,ho,wo} dy[n,ho,wo,k] * x[n, ho*st-pad+r, wo*st-pad+s, c];
 * db[k] = sum_{n,ho,wo} dy[n,ho,wo,k] (db may be NULL).  Both overwritten. */
void oracle_conv2d_backward_weight(const double* x, const double* dy, double* dw, double* db,
                                   int N, int H, int W, int C, int K, int R, int S, int stride, int pad)
{
    const int Ho = out_extent(H, R, stride, pad), Wo = out_extent(W, S, stride, pad);
    #pragma omp parallel for schedule(dynamic, 1)
    for (int k = 0; k < K; ++k) {
        double* dwk = dw + (size_t)k * R * S * C;
        for (size_t i = 0; i < (size_t)R * S * C; ++i) dwk[i] = 0.0;
        double bsum = 0.0;
        for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
            const double g = dy[(((size_t)n * Ho + ho) * Wo + wo) * K + k];
            bsum += g;
            for (int r = 0; r < R; ++r) {
                const int h = ho * stride - pad + r;
                if (h < 0 || h >= H) continue;
                for (int s = 0; s < S; ++s) {
                    const int wi = wo * stride - pad + s;
                    if (wi < 0 || wi >= W) continue;
                    const double* xp = x + (((size_t)n * H + h) * W + wi) * C;
                    double* dwp = dwk + ((size_t)r * S + s) * C;
                    for (int c = 0; c < C; ++c) dwp[c] += g * xp[c];
                }
            }
        }
        if (db) db[k] = bsum;
    }
}

/* Max pooling over k x k windows.  Out-of-range taps are skipped (they act as
 * -infinity).  arg[] receives the flat input-pixel index (h*W + w) of the first
 * maximum met in row-major window order. */
void oracle_maxpool_forward(const double* x, double* y, int32_t* arg,
                            int N, int H, int W, int C, int k, int stride, int pad)
{
    const int Ho = out_extent(H, k, stride, pad), Wo = out_extent(W, k, stride, pad);
    #pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
    for (int wo = 0; wo < Wo; ++wo)
    for (int c = 0; c < C; ++c) {
        int have = 0; double best = 0.0; int32_t where = -1;
        for (int r = 0; r < k; ++r) {
            const int h = ho * stride - pad + r;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < k; ++s) {
                const int wi = wo * stride - pad + s;
                if (wi < 0 || wi >= W) continue;
                const double v = x[(((size_t)n * H + h) * W + wi) * C + c];
                if (!have || v > best) { have = 1; best = v; where = h * W + wi; }
            }
        }
        const size_t o = (((size_t)n * Ho + ho) * Wo + wo) * C + c;
        y[o] = best; arg[o] = where;
    }
}

/* dx = scatter of dy to the recorded arg-max positions (overlapping windows add). */
void oracle_maxpool_backward(const double* dy, const int32_t* arg, double* dx,
                             int N, int H, int W, int C, int Ho, int Wo)
{
    memset(dx, 0, sizeof(double) * (size_t)N * H * W * C);
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
    for (int o = 0; o < Ho * Wo; ++o)
    for (int c = 0; c < C; ++c) {
        const size_t oi = ((size_t)n * Ho * Wo + o) * C + c;
        dx[((size_t)n * H * W + arg[oi]) * C + c] += dy[oi];
    }
}
