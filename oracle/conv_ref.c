/*
 * CPU oracle for the stride-1 forward convolution of a convolutional layer.
 *
 * TEST INFRASTRUCTURE ONLY: this file is the slow, plain definition the GPU
 * library is checked against. It shares no code with the GPU path, and only
 * the tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * What it computes (Section 2.1: each output element is the dot product of a
 * filter with a C x R x S sub-volume of the input, the sub-volume translated
 * over X and Y by the stride, with padding rows and columns added around the
 * input; Section 3: tensors are NCHW, X contiguous; Section 4: stride 1, fp32):
 *
 *   y[n,k,p,q] = sum_{c,r,s} xpad[n, c, p+r-pad_h, q+s-pad_w] * w[k,c,r,s]
 *   xpad = x inside [0,H) x [0,W), 0 outside
 *   P = H + 2*pad_h - R + 1,  Q = W + 2*pad_w - S + 1
 *
 * Readings where the text is silent: the filter is not flipped (the text
 * defines a dot product with the sub-volume whose top-left corner is the
 * output's position); padding cells hold zero; no bias, scaling or activation.
 *
 * Arithmetic: every product is formed in double (exact for two fp32 factors)
 * and added to a double accumulator, loops in the order n,k,p,q,c,r,s. A
 * second accumulator holds sum |x*w| over the same receptive field, which the
 * comparison tolerance is scaled by. No blocking, no reordering, no SIMD
 * intrinsics; threads split the (n,k) planes only.
 *
 * Parity status: pinned by tests/test_oracle_pins.py (hand-worked cases,
 * identity and shifted-delta filters, all-ones closed form, linearity,
 * matmul / im2col / per-tap decompositions, library cross-checks, operation
 * and touch counts).
 */
#include <math.h>
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
    const float *x, *w;
    double *y, *yabs;
    int N, C, H, W, K, R, S, pad_h, pad_w, P, Q;
    /* optional instrumentation (single-threaded only) */
    uint64_t *x_touch, *w_touch, *macs;
} conv_job_t;

/* One output element: the dot product over (c, r, s), padding taps skipped. */
static void conv_point(const conv_job_t *j, int n, int k, int p, int q, double *out, double *out_abs)
{
    double acc = 0.0, acc_abs = 0.0;
    for (int c = 0; c < j->C; ++c) {
        for (int r = 0; r < j->R; ++r) {
            for (int s = 0; s < j->S; ++s) {
                int h = p + r - j->pad_h;
                int v = q + s - j->pad_w;
                if (h < 0 || h >= j->H || v < 0 || v >= j->W)
                    continue; /* padding cell: contributes exactly zero */
                size_t xi = (((size_t)n * j->C + c) * j->H + h) * j->W + v;
                size_t wi = (((size_t)k * j->C + c) * j->R + r) * j->S + s;
                double prod = (double)j->x[xi] * (double)j->w[wi];
                acc += prod;
                acc_abs += fabs(prod);
                if (j->x_touch) j->x_touch[xi] += 1;
                if (j->w_touch) j->w_touch[wi] += 1;
                if (j->macs) *j->macs += 1;
            }
        }
    }
    *out = acc;
    if (out_abs) *out_abs = acc_abs;
}

static void conv_planes(const conv_job_t *j, long plane_begin, long plane_end)
{
    for (long nk = plane_begin; nk < plane_end; ++nk) {
        int n = (int)(nk / j->K), k = (int)(nk % j->K);
        for (int p = 0; p < j->P; ++p) {
            for (int q = 0; q < j->Q; ++q) {
                size_t yi = (((size_t)n * j->K + k) * j->P + p) * j->Q + q;
                conv_point(j, n, k, p, q, &j->y[yi], j->yabs ? &j->yabs[yi] : NULL);
            }
        }
    }
}

typedef struct {
    const conv_job_t *job;
    long begin, end;
} worker_arg_t;

static void *worker(void *arg)
{
    worker_arg_t *a = (worker_arg_t *)arg;
    conv_planes(a->job, a->begin, a->end);
    return NULL;
}

static int check_dims(int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0) return -2;
    if (pad_h < 0 || pad_w < 0) return -2;
    if (H + 2 * pad_h - R + 1 <= 0 || W + 2 * pad_w - S + 1 <= 0) return -3;
    return 0;
}

/*
 * Full layer. x, w: host fp32; y, yabs (may be NULL): host double [N][K][P][Q].
 * nthreads <= 0 means 1. Returns 0, or -1 null pointer, -2 bad dimension,
 * -3 empty output.
 */
int conv_ref(const float *x, const float *w, double *y, double *yabs,
             int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w, int nthreads)
{
    if (!x || !w || !y) return -1;
    int rc = check_dims(N, C, H, W, K, R, S, pad_h, pad_w);
    if (rc) return rc;
    conv_job_t job = {x, w, y, yabs, N, C, H, W, K, R, S, pad_h, pad_w,
                      H + 2 * pad_h - R + 1, W + 2 * pad_w - S + 1, NULL, NULL, NULL};
    long planes = (long)N * K;
    if (nthreads <= 1 || planes == 1) {
        conv_planes(&job, 0, planes);
        return 0;
    }
    if (nthreads > planes) nthreads = (int)planes;
    pthread_t *tid = (pthread_t *)malloc(sizeof(pthread_t) * nthreads);
    worker_arg_t *args = (worker_arg_t *)malloc(sizeof(worker_arg_t) * nthreads);
    for (int t = 0; t < nthreads; ++t) {
        args[t].job = &job;
        args[t].begin = planes * t / nthreads;
        args[t].end = planes * (t + 1) / nthreads;
        pthread_create(&tid[t], NULL, worker, &args[t]);
    }
    for (int t = 0; t < nthreads; ++t) pthread_join(tid[t], NULL);
    free(tid);
    free(args);
    return 0;
}

/*
 * Selected outputs only: coords holds npts quadruples (n,k,p,q); y and yabs
 * (may be NULL) receive npts doubles. Same arithmetic as conv_ref.
 */
int conv_ref_points(const float *x, const float *w, const int *coords, long npts, double *y, double *yabs,
                    int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w)
{
    if (!x || !w || !y || !coords) return -1;
    int rc = check_dims(N, C, H, W, K, R, S, pad_h, pad_w);
    if (rc) return rc;
    conv_job_t job = {x, w, NULL, NULL, N, C, H, W, K, R, S, pad_h, pad_w,
                      H + 2 * pad_h - R + 1, W + 2 * pad_w - S + 1, NULL, NULL, NULL};
    for (long i = 0; i < npts; ++i) {
        int n = coords[4 * i], k = coords[4 * i + 1], p = coords[4 * i + 2], q = coords[4 * i + 3];
        if (n < 0 || n >= N || k < 0 || k >= K || p < 0 || p >= job.P || q < 0 || q >= job.Q) return -2;
        conv_point(&job, n, k, p, q, &y[i], yabs ? &yabs[i] : NULL);
    }
    return 0;
}

/*
 * Full layer, single thread, with counters: x_touch[i] / w_touch[i] count the
 * multiply-adds that read element i of x / w, *macs counts all of them
 * (Section 3: a filter row is used once per output position, an interior input
 * row R*S times). Arrays must be zeroed by the caller; any may be NULL.
 */
int conv_ref_counted(const float *x, const float *w, double *y, uint64_t *x_touch, uint64_t *w_touch,
                     uint64_t *macs, int N, int C, int H, int W, int K, int R, int S, int pad_h, int pad_w)
{
    if (!x || !w || !y) return -1;
    int rc = check_dims(N, C, H, W, K, R, S, pad_h, pad_w);
    if (rc) return rc;
    conv_job_t job = {x, w, y, NULL, N, C, H, W, K, R, S, pad_h, pad_w,
                      H + 2 * pad_h - R + 1, W + 2 * pad_w - S + 1, x_touch, w_touch, macs};
    conv_planes(&job, 0, (long)N * K);
    return 0;
}
