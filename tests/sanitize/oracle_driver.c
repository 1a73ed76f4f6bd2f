/* Host sanitizer run of the C oracles (AddressSanitizer + UndefinedBehaviorSanitizer, gcc): a hand case and a few
 * ragged shapes through every entry point; any out-of-bounds access or undefined operation aborts the program.
 * Built and run by tests/test_sanitizers.py; test infrastructure only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_conv2d_f64(const double*, const double*, const double*, double*, int, int, int, int, int);
int oracle_conv2d_f64_at(const double*, const double*, const double*, const int64_t*, int64_t, double*, int, int, int, int, int);
int oracle_conv2d_general_f64(const double*, const double*, const double*, double*, int, int, int, int, int, int, int, int);

static double* filled(size_t n, unsigned seed) {
    double* p = malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) { seed = seed * 1664525u + 1013904223u; p[i] = (double)((int)(seed >> 24) - 128) / 64.0; }
    return p;
}

int main(void) {
    /* hand case: 3x3 image of ones, 3x3 filter of ones: the number of taps inside the image */
    double x[9], w[9], y[9];
    for (int i = 0; i < 9; ++i) x[i] = w[i] = 1.0;
    const double want[9] = {4, 6, 4, 6, 9, 6, 4, 6, 4};
    if (oracle_conv2d_f64(x, w, NULL, y, 1, 1, 3, 3, 1) != 0) return 2;
    for (int i = 0; i < 9; ++i) if (y[i] != want[i]) { printf("hand case differs at %d\n", i); return 3; }
    const int shapes[][5] = {{1, 1, 1, 1, 1}, {2, 3, 5, 7, 4}, {1, 5, 1, 9, 2}, {3, 2, 6, 1, 3}, {1, 4, 8, 8, 5}};   /* N C H W K */
    for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s) {
        const int N = shapes[s][0], C = shapes[s][1], H = shapes[s][2], W = shapes[s][3], K = shapes[s][4];
        double *xx = filled((size_t)N * C * H * W, 1 + s), *ww = filled((size_t)K * C * 9, 7 + s), *bb = filled(K, 11 + s);
        double* yy = malloc((size_t)N * K * H * W * sizeof(double));
        if (oracle_conv2d_f64(xx, ww, bb, yy, N, C, H, W, K) != 0) return 4;
        /* every element once more through the one-output-at-a-time variant */
        const int64_t total = (int64_t)N * K * H * W;
        int64_t* idx = malloc(total * sizeof(int64_t));
        double* at = malloc(total * sizeof(double));
        for (int64_t i = 0; i < total; ++i) idx[i] = total - 1 - i;
        if (oracle_conv2d_f64_at(xx, ww, bb, idx, total, at, N, C, H, W, K) != 0) return 5;
        for (int64_t i = 0; i < total; ++i) if (fabs(at[i] - yy[total - 1 - i]) > 1e-12) { printf("at-variant differs\n"); return 6; }
        /* the general oracle: R = 3 stride 1 pad 1 is the same operator; stride 2 and 1x1 run for bounds only */
        double* yg = malloc((size_t)N * K * H * W * sizeof(double));
        if (oracle_conv2d_general_f64(xx, ww, bb, yg, N, C, H, W, K, 3, 1, 1) != 0) return 7;
        for (int64_t i = 0; i < total; ++i) if (fabs(yg[i] - yy[i]) > 1e-12) { printf("general oracle differs\n"); return 8; }
        if (oracle_conv2d_general_f64(xx, ww, bb, yg, N, C, H, W, K, 3, 2, 1) != 0) return 9;
        double* w1 = filled((size_t)K * C, 13 + s);
        if (oracle_conv2d_general_f64(xx, w1, NULL, yg, N, C, H, W, K, 1, 1, 0) != 0) return 10;
        free(xx); free(ww); free(bb); free(yy); free(idx); free(at); free(yg); free(w1);
    }
    /* bad arguments are refused, not dereferenced */
    if (oracle_conv2d_f64(NULL, w, NULL, y, 1, 1, 3, 3, 1) == 0) return 11;
    if (oracle_conv2d_f64(x, w, NULL, y, 0, 1, 3, 3, 1) == 0) return 12;
    printf("oracle sanitizer run ok\n");
    return 0;
}
