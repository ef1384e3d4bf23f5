/* Driver for the sanitizer build of the oracle (address + undefined behaviour): runs conv_ref, conv_ref_points and
 * conv_ref_counted on small layers with every kind of edge (padding wider than the filter, 1x1 maps, non-square
 * filters, several threads) and checks two closed forms, so that the run also fails on wrong answers. */
#include <stdio.h>
#include <stdlib.h>

int conv_ref(const float *x, const float *w, double *y, double *yabs, int N, int C, int H, int W, int K, int R, int S,
             int pad_h, int pad_w, int nthreads);
int conv_ref_points(const float *x, const float *w, const int *coords, long npts, double *y, double *yabs, int N, int C,
                    int H, int W, int K, int R, int S, int pad_h, int pad_w);
int conv_ref_counted(const float *x, const float *w, double *y, unsigned long long *x_touch, unsigned long long *w_touch,
                     unsigned long long *macs, int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w);

static const int SHAPES[][9] = {
    {1, 1, 3, 3, 1, 2, 2, 0, 0}, {2, 3, 5, 7, 4, 3, 3, 1, 1}, {1, 2, 1, 1, 3, 3, 3, 1, 1}, {3, 4, 6, 5, 2, 1, 5, 0, 2},
    {1, 5, 4, 4, 7, 5, 5, 4, 4}, {2, 8, 9, 9, 5, 1, 1, 0, 0}, {1, 1, 2, 9, 1, 2, 3, 1, 0}, {4, 2, 3, 3, 2, 3, 3, 2, 2},
};

int main(void)
{
    int bad = 0;
    for (unsigned i = 0; i < sizeof(SHAPES) / sizeof(SHAPES[0]); ++i) {
        const int *d = SHAPES[i];
        const int N = d[0], C = d[1], H = d[2], W = d[3], K = d[4], R = d[5], S = d[6], ph = d[7], pw = d[8];
        const int P = H + 2 * ph - R + 1, Q = W + 2 * pw - S + 1;
        const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * C * R * S, ny = (size_t)N * K * P * Q;
        float *x = malloc(nx * sizeof(float)), *w = malloc(nw * sizeof(float));
        double *y = malloc(ny * sizeof(double)), *ya = malloc(ny * sizeof(double)), *y2 = malloc(ny * sizeof(double));
        unsigned long long *xt = calloc(nx, sizeof(*xt)), *wt = calloc(nw, sizeof(*wt)), macs = 0;
        int *coords = malloc(ny * 4 * sizeof(int));
        for (size_t e = 0; e < nx; ++e) x[e] = 1.0f;
        for (size_t e = 0; e < nw; ++e) w[e] = 1.0f;
        for (int threads = 1; threads <= 5; threads += 2)
            if (conv_ref(x, w, y, ya, N, C, H, W, K, R, S, ph, pw, threads) != 0) ++bad;
        /* all ones: every output counts its in-bounds taps, C * rows * columns */
        size_t e = 0;
        for (int n = 0; n < N; ++n)
            for (int k = 0; k < K; ++k)
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < Q; ++q, ++e) {
                        int rows = 0, cols = 0;
                        for (int r = 0; r < R; ++r) rows += p + r - ph >= 0 && p + r - ph < H;
                        for (int s = 0; s < S; ++s) cols += q + s - pw >= 0 && q + s - pw < W;
                        if (y[e] != (double)C * rows * cols || ya[e] != y[e]) ++bad;
                        coords[4 * e] = n; coords[4 * e + 1] = k; coords[4 * e + 2] = p; coords[4 * e + 3] = q;
                    }
        if (conv_ref_points(x, w, coords, (long)ny, y2, ya, N, C, H, W, K, R, S, ph, pw) != 0) ++bad;
        for (e = 0; e < ny; ++e) bad += y2[e] != y[e];
        if (conv_ref_counted(x, w, y2, xt, wt, &macs, N, C, H, W, K, R, S, ph, pw) != 0) ++bad;
        double total = 0;
        for (e = 0; e < ny; ++e) total += y[e];
        if ((double)macs != total) ++bad; /* with all ones every multiply-add adds one */
        free(x); free(w); free(y); free(ya); free(y2); free(xt); free(wt); free(coords);
    }
    /* argument errors are codes */
    double one;
    float f = 1.0f;
    if (conv_ref(NULL, &f, &one, &one, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1) != -1) ++bad;
    if (conv_ref(&f, &f, &one, &one, 0, 1, 1, 1, 1, 1, 1, 0, 0, 1) != -2) ++bad;
    if (conv_ref(&f, &f, &one, &one, 1, 1, 1, 1, 1, 3, 3, 0, 0, 1) != -3) ++bad;
    printf("oracle under sanitizers: %d problems\n", bad);
    return bad != 0;
}
