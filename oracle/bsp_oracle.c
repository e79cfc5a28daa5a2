/*
 * CPU oracle for block-sparse convolution / fully-connected inference.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against; the product path never calls it and shares
 * no code with it.
 *
 * What it computes (paper, Section I: Y = W*X + b with Y of size M x N x O,
 * X of size L x J x I, W of size O x H x K x I, b of size O; a leading batch
 * dimension is added here):
 *
 *   Y[n,m,q,o] = b[o] + sum_{h<H} sum_{k<K} sum_{i<I}
 *                  Wm[o,h,k,i] * X[n, m*sh + h - ph, q*sw + k - pw, i]
 *
 * with X taken as zero outside [0,L) x [0,J), cross-correlation (no kernel
 * flip), output size floor((L + 2ph - H)/sh) + 1.  Wm is the weight tensor
 * with the block mask of Eq. (1) already applied by the caller: this routine
 * is the ordinary dense definition and skips nothing.  A fully-connected
 * layer is the case H = K = L = J = 1 (Section III: a GEMM is a 1x1
 * convolution).
 *
 * Everything is double precision and accumulated in exactly the loop order
 * written above (h, then k, then i), one scalar at a time.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double one_output(const double *X, const double *Wm, const double *bias,
                         int64_t n, int64_t m, int64_t q, int64_t o,
                         int64_t L, int64_t J, int64_t I,
                         int64_t H, int64_t K,
                         int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    double acc = bias ? bias[o] : 0.0;
    for (int64_t h = 0; h < H; ++h) {
        int64_t y = m * sh + h - ph;
        if (y < 0 || y >= L)
            continue;                      /* zero padding rows add nothing */
        for (int64_t k = 0; k < K; ++k) {
            int64_t x = q * sw + k - pw;
            if (x < 0 || x >= J)
                continue;
            const double *xp = X + ((n * L + y) * J + x) * I;
            const double *wp = Wm + ((o * H + h) * K + k) * I;
            for (int64_t i = 0; i < I; ++i)
                acc += wp[i] * xp[i];
        }
    }
    return acc;
}

/* Full output tensor, NHWC in, NHWC out.  Returns the number of threads used. */
int oracle_conv2d(const double *X, const double *Wm, const double *bias,
                  double *Y, int64_t B, int64_t L, int64_t J, int64_t I,
                  int64_t O, int64_t H, int64_t K,
                  int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                  int nthreads)
{
    int64_t M = (L + 2 * ph - H) / sh + 1;
    int64_t N = (J + 2 * pw - K) / sw + 1;
    int used = 1;
    if (M < 1 || N < 1)
        return -1;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
    used = omp_get_max_threads();
#else
    (void)nthreads;
#endif
    int64_t rows = B * M;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t n = r / M, m = r % M;
        for (int64_t q = 0; q < N; ++q)
            for (int64_t o = 0; o < O; ++o)
                Y[((n * M + m) * N + q) * O + o] =
                    one_output(X, Wm, bias, n, m, q, o, L, J, I, H, K,
                               sh, sw, ph, pw);
    }
    return used;
}

/* Selected outputs only: pos is [npos][4] = (n, m, q, o).  */
int oracle_conv2d_at(const double *X, const double *Wm, const double *bias,
                     const int64_t *pos, int64_t npos, double *out,
                     int64_t B, int64_t L, int64_t J, int64_t I,
                     int64_t O, int64_t H, int64_t K,
                     int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    int64_t M = (L + 2 * ph - H) / sh + 1;
    int64_t N = (J + 2 * pw - K) / sw + 1;
    if (M < 1 || N < 1)
        return -1;
    for (int64_t t = 0; t < npos; ++t) {
        int64_t n = pos[4 * t], m = pos[4 * t + 1];
        int64_t q = pos[4 * t + 2], o = pos[4 * t + 3];
        if (n < 0 || n >= B || m < 0 || m >= M || q < 0 || q >= N ||
            o < 0 || o >= O)
            return -2;
        out[t] = one_output(X, Wm, bias, n, m, q, o, L, J, I, H, K,
                            sh, sw, ph, pw);
    }
    return 0;
}
