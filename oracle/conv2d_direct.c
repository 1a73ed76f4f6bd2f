/*
 * ORACLE — TEST INFRASTRUCTURE ONLY.  Not part of the product path: nothing in
 * the library, its Python binding or its kernels may include, link or call this.
 *
 * Plain fp64 direct 2-D cross-correlation, 3x3 filter, stride 1, zero padding 1.
 * This is the definition of the operator the paper's Winograd path replaces
 * (the 2-D convolution operator of Section "Techniques"; tensor shapes as in the
 * header of Table 1: filter [KW,KH,IC,OC], activation [IW,IH,IC,N], fastest
 * dimension first, i.e. memory order w[K][C][3][3], x[N][C][H][W]).
 *
 *   y[n,k,i,j] = bias[k] + sum_{c,r,s} xhat[n,c,i+r-1,j+s-1] * w[k,c,r,s]
 *   xhat = x inside the image, 0 outside.
 *
 * The Winograd algorithm reaches exactly this result (up to rounding), so the
 * oracle is the definition itself, written out.  No blocking, no fusion.
 */
#include <stddef.h>
#include <stdint.h>

/* Whole tensor.  bias may be NULL (treated as zero).  Returns 0, or -1 on bad sizes. */
int oracle_conv2d_f64(const double *x, const double *w, const double *bias, double *y,
                      int N, int C, int H, int W, int K)
{
    if (!x || !w || !y || N < 1 || C < 1 || H < 1 || W < 1 || K < 1) return -1;
    const size_t plane = (size_t)H * (size_t)W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            double *yp = y + ((size_t)n * K + k) * plane;
            const double b = bias ? bias[k] : 0.0;
            for (size_t p = 0; p < plane; ++p) yp[p] = b;
            for (int c = 0; c < C; ++c) {
                const double *xp = x + ((size_t)n * C + c) * plane;
                const double *wp = w + ((size_t)k * C + c) * 9;
                for (int r = 0; r < 3; ++r) {
                    for (int s = 0; s < 3; ++s) {
                        const double wv = wp[r * 3 + s];
                        /* output (i,j) reads input (i+r-1, j+s-1); keep only in-image taps */
                        const int i0 = (r == 0) ? 1 : 0, i1 = (r == 2) ? H - 1 : H;
                        const int j0 = (s == 0) ? 1 : 0, j1 = (s == 2) ? W - 1 : W;
                        for (int i = i0; i < i1; ++i) {
                            const double *xr = xp + (size_t)(i + r - 1) * W + (s - 1);
                            double *yr = yp + (size_t)i * W;
                            for (int j = j0; j < j1; ++j) yr[j] += xr[j] * wv;
                        }
                    }
                }
            }
        }
    }
    return 0;
}

/*
 * Selected outputs only: idx[q] is the flat index into y[N][K][H][W]; out[q] gets
 * that element.  Written as the defining sum with explicit bounds tests, one
 * output at a time, so full-size layers can be spot-checked.
 */
int oracle_conv2d_f64_at(const double *x, const double *w, const double *bias,
                         const int64_t *idx, int64_t n_idx, double *out,
                         int N, int C, int H, int W, int K)
{
    if (!x || !w || !idx || !out || N < 1 || C < 1 || H < 1 || W < 1 || K < 1) return -1;
    const int64_t total = (int64_t)N * K * H * W;
    for (int64_t q = 0; q < n_idx; ++q)
        if (idx[q] < 0 || idx[q] >= total) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < n_idx; ++q) {
        int64_t f = idx[q];
        const int j = (int)(f % W); f /= W;
        const int i = (int)(f % H); f /= H;
        const int k = (int)(f % K); f /= K;
        const int n = (int)f;
        double acc = bias ? bias[k] : 0.0;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < 3; ++r)
                for (int s = 0; s < 3; ++s) {
                    const int ii = i + r - 1, jj = j + s - 1;
                    if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                    acc += x[(((size_t)n * C + c) * H + ii) * W + jj] *
                           w[(((size_t)k * C + c) * 3 + r) * 3 + s];
                }
        out[q] = acc;
    }
    return 0;
}

int oracle_num_threads(void);
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
