/* Runs every entry point of the CPU oracle on small, awkward shapes (non-square planes, different strides and
 * paddings per axis, a single image, map length 1, top-k equal to the map length, all three element types and all
 * three filter-gradient layouts).  Built with -fsanitize=address,undefined by tests/test_oracle_sanitized.py: an
 * out-of-bounds index, a signed overflow or a misaligned access anywhere in the oracle aborts the run.  The values
 * are not checked here (the pins in tests/test_oracle_*.py do that); the outputs are only summed so that nothing
 * is optimised away. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct { int32_t N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w; } oracle_shape;
int oracle_out_h(const oracle_shape *);
int oracle_out_w(const oracle_shape *);
int oracle_wgrad_exact(const oracle_shape *, const void *, const void *, int, double *);
int oracle_wgrad_exact_at(const oracle_shape *, const void *, const void *, int, const int64_t *, int64_t, double *);
int oracle_select(const oracle_shape *, const void *, int, int32_t *, double *);
int oracle_wgrad_approx(const oracle_shape *, const void *, const void *, int, double, double *, int32_t *, double *);
int oracle_select_topk(const oracle_shape *, const void *, int, int, int32_t *, double *);
int oracle_wgrad_approx_topk(const oracle_shape *, const void *, const void *, int, int, double, double *, int32_t *, double *);
int oracle_wgrad_exact_nhwc(const oracle_shape *, const void *, const void *, int, int, double *);
int oracle_wgrad_approx_nhwc(const oracle_shape *, const void *, const void *, int, int, double, double *, int32_t *, double *);
void oracle_philox4x32_10(const uint32_t *, const uint32_t *, uint32_t *);
void oracle_random_normal(uint64_t, uint64_t, int64_t, double, double *);

static uint32_t lcg = 12345u;
static double next_value(void) { lcg = lcg * 1664525u + 1013904223u; return ((int)(lcg >> 9) % 2001 - 1000) / 1000.0; }

static double run_shape(oracle_shape g, int dtype)
{
    const int Ho = oracle_out_h(&g), Wo = oracle_out_w(&g), len = Ho * Wo;
    const size_t nx = (size_t)g.N * g.C * g.H * g.W, ny = (size_t)g.N * g.K * len, nw = (size_t)g.K * g.C * g.R * g.S;
    const size_t esz = dtype == 2 ? 8 : (dtype == 0 ? 4 : 2);
    /* exact-size allocations: the sanitizer sees one element too far */
    void *X = malloc(nx * esz), *dY = malloc(ny * esz);
    for (size_t i = 0; i < nx + ny; ++i) {
        const double v = next_value();
        void *dst = i < nx ? X : dY;
        const size_t j = i < nx ? i : i - nx;
        if (dtype == 2) ((double *)dst)[j] = v;
        else if (dtype == 0) ((float *)dst)[j] = (float)v;
        else { float f = (float)v; uint32_t b; __builtin_memcpy(&b, &f, 4); ((uint16_t *)dst)[j] = (uint16_t)(b >> 16); }
    }
    double *dW = malloc(nw * sizeof(double)), *S = malloc((size_t)g.N * g.K * sizeof(double));
    int32_t *idx = malloc((size_t)g.N * g.K * (size_t)(len < 64 ? len : 64) * sizeof(int32_t));
    double sum = 0;
    if (oracle_wgrad_exact(&g, X, dY, dtype, dW)) exit(2);
    for (size_t i = 0; i < nw; ++i) sum += dW[i];
    int64_t at[3] = {0, (int64_t)nw - 1, (int64_t)nw / 2};
    double got[3];
    if (oracle_wgrad_exact_at(&g, X, dY, dtype, at, 3, got)) exit(2);
    sum += got[0] + got[1] + got[2];
    if (oracle_select(&g, dY, dtype, idx, S)) exit(2);
    if (oracle_wgrad_approx(&g, X, dY, dtype, 0.5, dW, idx, S)) exit(2);
    for (size_t i = 0; i < nw; ++i) sum += dW[i];
    if (oracle_wgrad_approx(&g, X, dY, dtype, 1.0, dW, NULL, NULL)) exit(2);
    const int ks[3] = {1, len < 3 ? len : 3, len < 64 ? len : 64};
    for (int t = 0; t < 3; ++t) {
        if (oracle_select_topk(&g, dY, dtype, ks[t], idx, S)) exit(2);
        if (oracle_wgrad_approx_topk(&g, X, dY, dtype, ks[t], 2.0, dW, idx, S)) exit(2);
        for (size_t i = 0; i < nw; ++i) sum += dW[i];
    }
    for (int layout = 0; layout < 3; ++layout) {            /* the same bytes read as [N,H,W,C]: sizes agree */
        if (oracle_wgrad_exact_nhwc(&g, X, dY, dtype, layout, dW)) exit(2);
        if (oracle_wgrad_approx_nhwc(&g, X, dY, dtype, layout, 1.0, dW, idx, S)) exit(2);
        for (size_t i = 0; i < nw; ++i) sum += dW[i];
    }
    free(X); free(dY); free(dW); free(S); free(idx);
    return sum;
}

int main(void)
{
    const oracle_shape shapes[] = {
        {2, 3, 5, 7, 4, 3, 3, 1, 1, 1, 1},      /* non-square plane                                   */
        {3, 2, 9, 6, 5, 3, 2, 2, 1, 1, 0},      /* different filter extents, strides and paddings      */
        {1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0},      /* everything of size one: map length 1                */
        {2, 4, 2, 2, 3, 3, 3, 1, 1, 1, 1},      /* 2x2 planes: most taps fall into the padding         */
        {2, 2, 8, 8, 2, 5, 5, 3, 3, 2, 2},      /* wide filter, stride 3                               */
        {4, 1, 4, 10, 2, 1, 4, 1, 2, 0, 3},     /* padding wider than the filter reaches               */
    };
    double sum = 0;
    for (unsigned i = 0; i < sizeof shapes / sizeof shapes[0]; ++i)
        for (int dtype = 0; dtype < 3; ++dtype) sum += run_shape(shapes[i], dtype);
    const uint32_t ctr[4] = {1u, 2u, 3u, 4u}, key[2] = {5u, 6u};
    uint32_t w[4];
    oracle_philox4x32_10(ctr, key, w);
    double r[37];
    oracle_random_normal(0x123456789abcdefull, 0xfffffffffffffff0ull, 37, 1.0 / 128, r);   /* the offset wraps in 64 bits */
    for (int i = 0; i < 37; ++i) sum += r[i];
    printf("oracle sanitize run ok (%u words, checksum %.6g)\n", w[0] ^ w[1] ^ w[2] ^ w[3], sum);
    return 0;
}
