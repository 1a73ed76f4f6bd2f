/*
 * ORACLE — TEST INFRASTRUCTURE ONLY.  Not part of the product path: nothing in
 * the library, its Python binding or its kernels may include, link or call this.
 *
 * Plain fp64 direct 2-D cross-correlation with a square R x R filter, stride st
 * and symmetric zero padding `pad`: the other convolution flavours a Stable-
 * Diffusion UNet and VAE call besides the 3x3 / stride-1 one (1x1 projections,
 * 3x3 / stride-2 down-sampling).  The paper's Section "Techniques" speaks of the
 * 2-D convolution operator in general and defines none of them; the textbook
 * definition is written out, one output element at a time, with explicit bounds
 * tests:
 *
 *   Ho = (H + 2 pad - R) / st + 1,  Wo likewise
 *   y[n,k,i,j] = bias[k] + sum_{c,r,s} xhat[n, c, i*st + r - pad, j*st + s - pad] * w[k,c,r,s]
 *   xhat = x inside the image, 0 outside.
 *
 * Memory order x[N][C][H][W], w[K][C][R][R], y[N][K][Ho][Wo].
 */
#include <stddef.h>

int oracle_conv2d_general_f64(const double *x, const double *w, const double *bias, double *y,
                              int N, int C, int H, int W, int K, int R, int st, int pad)
{
    if (!x || !w || !y || N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || st < 1 || pad < 0) return -1;
    if (H + 2 * pad < R || W + 2 * pad < R) return -1;
    const int Ho = (H + 2 * pad - R) / st + 1, Wo = (W + 2 * pad - R) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int i = 0; i < Ho; ++i) {
                for (int j = 0; j < Wo; ++j) {
                    double acc = bias ? bias[k] : 0.0;
                    for (int c = 0; c < C; ++c) {
                        for (int r = 0; r < R; ++r) {
                            const int ii = i * st + r - pad;
                            if (ii < 0 || ii >= H) continue;
                            for (int s = 0; s < R; ++s) {
                                const int jj = j * st + s - pad;
                                if (jj < 0 || jj >= W) continue;
                                acc += x[(((size_t)n * C + c) * H + ii) * W + jj] *
                                       w[(((size_t)k * C + c) * R + r) * R + s];
                            }
                        }
                    }
                    y[(((size_t)n * K + k) * Ho + i) * Wo + j] = acc;
                }
            }
        }
    }
    return 0;
}
