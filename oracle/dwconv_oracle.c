/*
 * dwconv_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct CPU definition of the depthwise 1-D
 * convolution operator and its two gradients, written straight from the
 * operator definition of the paper (Sec. IV-A "Common Problem Definition and
 * Memory Layout": eq. (dwconv) forward, eq. (dx_def) input gradient,
 * eq. (dk_def) kernel gradient).  Every product is formed and accumulated in
 * fp64 in natural index order; there is no blocking, fusion or reordering.
 *
 * This file shares nothing with the HIP library: no headers, no helpers, no
 * constants.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  The product path never does.
 *
 * Layout (Sec. IV-A): x, y, dy, dx are dense row-major [B, C, L] (t is the
 * stride-1 index); w, dw are dense row-major [C, K].  The paper calls the
 * channel count H and the filter k; here they are C and w.
 *
 * Padding: the paper fixes p = floor(K/2) (eq. (padding_width)).  The oracle
 * takes p = pad_left in [0, K-1] as an argument; the output length is always
 * L and x~ (zero-padded x) is zero outside [0, L).  p = floor(K/2) is the
 * paper's case, p = K-1 is causal.
 *
 * Every routine returns, next to each value, the sum of the absolute values
 * of the same terms ("abs" arrays).  Tests normalise GPU-vs-oracle error by
 * it.
 *
 * Pins (tests/test_oracle_pins.py, CPU only): identity filter and delta input
 * closed forms, all-ones tap counts, a hand-worked example, a scatter-form
 * brute force, fp64 grouped conv1d of a library and its autograd, finite
 * differences, and the adjoint identity <dY, fwd(x,w)> = <dX, x> = <dW, w>.
 */
#include <math.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the parallel loops below will use. */
int dwconv_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Forward, eq. (dwconv):
 *     y[b,c,t] = sum_{j=0}^{K-1} x~[b,c,t+j-p] * w[c,j]
 * Cross-correlation: the filter is not flipped.
 * Rows (b,c) are independent; each is produced by one thread in fixed order.
 */
int dwconv_oracle_fwd(const float *x, const float *w, double *y, double *yabs,
                      long B, long C, long L, long K, long p)
{
    if (!x || !w || !y || !yabs) return 1;
    if (B < 1 || C < 1 || L < 1 || K < 1) return 2;
    if (p < 0 || p > K - 1) return 3;
    long rows = B * C;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        long c = r % C;
        const float *xr = x + (size_t)r * (size_t)L;
        const float *wc = w + (size_t)c * (size_t)K;
        for (long t = 0; t < L; ++t) {
            double s = 0.0, a = 0.0;
            for (long j = 0; j < K; ++j) {
                long u = t + j - p;
                if (u < 0 || u >= L) continue;       /* x~ is zero there */
                double term = (double)xr[u] * (double)wc[j];
                s += term;
                a += fabs(term);
            }
            y[(size_t)r * (size_t)L + (size_t)t] = s;
            yabs[(size_t)r * (size_t)L + (size_t)t] = a;
        }
    }
    return 0;
}

/*
 * Input gradient: the adjoint of eq. (dwconv) with respect to x.
 * y[t] receives x[s] * w[j] exactly when s = t + j - p, i.e. t = s - j + p, so
 *     dx[b,c,s] = sum_{j=0}^{K-1} dy~[b,c,s-j+p] * w[c,j].
 * Substituting j -> K-1-j gives sum_j dy~[s+j-(K-1-p)] * w[K-1-j], which is
 * the printed eq. (dx_def) when K-1-p = p (odd K).  For even K the printed
 * offset differs by one from the adjoint; the adjoint is what is computed
 * here (it is the gradient, and it is what the paper's own validation against
 * autograd requires).
 */
int dwconv_oracle_bwd_input(const float *dy, const float *w, double *dx,
                            double *dxabs, long B, long C, long L, long K,
                            long p)
{
    if (!dy || !w || !dx || !dxabs) return 1;
    if (B < 1 || C < 1 || L < 1 || K < 1) return 2;
    if (p < 0 || p > K - 1) return 3;
    long rows = B * C;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        long c = r % C;
        const float *gr = dy + (size_t)r * (size_t)L;
        const float *wc = w + (size_t)c * (size_t)K;
        for (long s = 0; s < L; ++s) {
            double acc = 0.0, a = 0.0;
            for (long j = 0; j < K; ++j) {
                long t = s - j + p;
                if (t < 0 || t >= L) continue;       /* no such output */
                double term = (double)gr[t] * (double)wc[j];
                acc += term;
                a += fabs(term);
            }
            dx[(size_t)r * (size_t)L + (size_t)s] = acc;
            dxabs[(size_t)r * (size_t)L + (size_t)s] = a;
        }
    }
    return 0;
}

/*
 * Kernel (weight) gradient, eq. (dk_def):
 *     dw[c,j] = sum_{b=0}^{B-1} sum_{t=0}^{L-1} dy[b,c,t] * x~[b,c,t+j-p]
 * Channels are independent; each coefficient is summed by one thread, b outer,
 * t inner.
 */
int dwconv_oracle_bwd_weight(const float *x, const float *dy, double *dw,
                             double *dwabs, long B, long C, long L, long K,
                             long p)
{
    if (!x || !dy || !dw || !dwabs) return 1;
    if (B < 1 || C < 1 || L < 1 || K < 1) return 2;
    if (p < 0 || p > K - 1) return 3;
    long coeffs = C * K;
#pragma omp parallel for schedule(dynamic, 16)
    for (long q = 0; q < coeffs; ++q) {
        long c = q / K;
        long j = q % K;
        double acc = 0.0, a = 0.0;
        for (long b = 0; b < B; ++b) {
            const float *xr = x + ((size_t)b * (size_t)C + (size_t)c) * (size_t)L;
            const float *gr = dy + ((size_t)b * (size_t)C + (size_t)c) * (size_t)L;
            for (long t = 0; t < L; ++t) {
                long u = t + j - p;
                if (u < 0 || u >= L) continue;       /* x~ is zero there */
                double term = (double)gr[t] * (double)xr[u];
                acc += term;
                a += fabs(term);
            }
        }
        dw[q] = acc;
        dwabs[q] = a;
    }
    return 0;
}
