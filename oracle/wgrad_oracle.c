/*
 * CPU oracle for the filter (weight) gradient of a convolution layer, exact and
 * in the "Max Gradient Approximation" form of arXiv 1908.05460.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64
 * implementation written from the paper so that a reader can check it by eye:
 * no blocking, no fusion, no reordering beyond what the definition states.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * load it.  It shares no code, header or table with the HIP library.
 *
 * Notation.  The paper writes I (input activations, NCHW), dO (output
 * gradient, NCHW), df (filter gradient) and uses K for the filter size
 * (Section 2.4).  Here: X = I  [N,C,H,W],  dY = dO  [N,K,Ho,Wo],
 * dW = df  [K,C,R,S]  (K = number of output channels, R x S = filter size),
 * Ho = floor((H + 2*pad_h - R)/stride_h) + 1, likewise Wo.
 *
 * Pins (tests/test_oracle_*.py): the exact gradient is pinned by the identity
 * dW[k,c,r,s] = L(e_kcrs) with L(W) = sum(dY * conv(X, W)) evaluated through an
 * independently written forward convolution, by the 1x1 case reducing to a
 * library GEMM, by a library autograd, by bilinearity and by stride/upsample
 * equivalence.  The selection is pinned by brute force and crafted ties.  The
 * approximation is pinned by "approx(X,dY) == exact(X, sparsify(dY))"
 * (Section 2.4: with one retained element per map the convolution becomes a
 * collection of patches), by the single-non-zero case, by the constant-input
 * closed form and by homogeneity.  The random generator is pinned by the
 * published known-answer vectors of Philox4x32-10 and by sample moments.
 * The paper prints no worked numerical example (its Figure 2 is an image), so
 * no value in the tests comes from the paper itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t N, C, H, W;     /* X  : [N,C,H,W]                              */
    int32_t K, R, S;        /* dW : [K,C,R,S]                              */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
} oracle_shape;

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

static int out_h(const oracle_shape *g) { return (g->H + 2 * g->pad_h - g->R) / g->stride_h + 1; }
static int out_w(const oracle_shape *g) { return (g->W + 2 * g->pad_w - g->S) / g->stride_w + 1; }

int oracle_out_h(const oracle_shape *g) { return out_h(g); }
int oracle_out_w(const oracle_shape *g) { return out_w(g); }

/* Exact upcast of `count` elements to double.  bf16 is the upper half of an
 * IEEE binary32, so widening it is a 16-bit shift; nothing is rounded. */
static double *to_double(const void *src, int dtype, size_t count)
{
    double *dst = (double *)malloc((count ? count : 1) * sizeof(double));
    if (!dst) return NULL;
    if (dtype == ORACLE_F64) {
        memcpy(dst, src, count * sizeof(double));
    } else if (dtype == ORACLE_F32) {
        const float *s = (const float *)src;
        for (size_t i = 0; i < count; ++i) dst[i] = (double)s[i];
    } else {
        const uint16_t *s = (const uint16_t *)src;
        for (size_t i = 0; i < count; ++i) {
            uint32_t bits = (uint32_t)s[i] << 16;
            float f;
            memcpy(&f, &bits, sizeof f);
            dst[i] = (double)f;
        }
    }
    return dst;
}

/* X with zero padding: the value the convolution sees at input row ih, col iw. */
static double x_at(const double *X, const oracle_shape *g, int n, int c, int ih, int iw)
{
    if (ih < 0 || ih >= g->H || iw < 0 || iw >= g->W) return 0.0;
    return X[(((size_t)n * g->C + c) * g->H + ih) * g->W + iw];
}

/* One entry of the exact filter gradient (Section 2.4: df is I convolved with dO):
 *   dW[k,c,r,s] = sum_{n,h,w} dY[n,k,h,w] * X[n,c,h*stride_h + r - pad_h, w*stride_w + s - pad_w]
 * summed in the order n, h, w as written. */
static double exact_entry(const oracle_shape *g, const double *X, const double *dY,
                          int k, int c, int r, int s)
{
    const int Ho = out_h(g), Wo = out_w(g);
    double acc = 0.0;
    for (int n = 0; n < g->N; ++n)
        for (int h = 0; h < Ho; ++h)
            for (int w = 0; w < Wo; ++w) {
                double dy = dY[(((size_t)n * g->K + k) * Ho + h) * Wo + w];
                acc += dy * x_at(X, g, n, c, h * g->stride_h + r - g->pad_h,
                                 w * g->stride_w + s - g->pad_w);
            }
    return acc;
}

/* Exact dW for every (k,c,r,s).  dW is [K,C,R,S] in double. Returns 0, or -1 on
 * allocation failure. */
int oracle_wgrad_exact(const oracle_shape *g, const void *X_, const void *dY_, int dtype,
                       double *dW)
{
    const int Ho = out_h(g), Wo = out_w(g);
    double *X = to_double(X_, dtype, (size_t)g->N * g->C * g->H * g->W);
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * Ho * Wo);
    if (!X || !dY) { free(X); free(dY); return -1; }
    const long total = (long)g->K * g->C * g->R * g->S;
#pragma omp parallel for schedule(static)
    for (long o = 0; o < total; ++o) {
        int s = (int)(o % g->S);
        int r = (int)((o / g->S) % g->R);
        int c = (int)((o / ((long)g->S * g->R)) % g->C);
        int k = (int)(o / ((long)g->S * g->R * g->C));
        dW[o] = exact_entry(g, X, dY, k, c, r, s);
    }
    free(X); free(dY);
    return 0;
}

/* Exact dW at `count` chosen flat indices o = ((k*C + c)*R + r)*S + s only; used
 * to check full-size layers entry by entry without computing all of dW. */
int oracle_wgrad_exact_at(const oracle_shape *g, const void *X_, const void *dY_, int dtype,
                          const int64_t *flat, int64_t count, double *out)
{
    const int Ho = out_h(g), Wo = out_w(g);
    double *X = to_double(X_, dtype, (size_t)g->N * g->C * g->H * g->W);
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * Ho * Wo);
    if (!X || !dY) { free(X); free(dY); return -1; }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < count; ++i) {
        int64_t o = flat[i];
        int s = (int)(o % g->S);
        int r = (int)((o / g->S) % g->R);
        int c = (int)((o / ((int64_t)g->S * g->R)) % g->C);
        int k = (int)(o / ((int64_t)g->S * g->R * g->C));
        out[i] = exact_entry(g, X, dY, k, c, r, s);
    }
    free(X); free(dY);
    return 0;
}

/* Magnitude used for ranking the positions of a map.  Algorithm 1 says nothing
 * about NaN; the rule of this build: a NaN ranks as magnitude zero, i.e. it ties
 * with the zeros of the map and the lowest position among them wins. */
static double rank_magnitude(double v)
{
    double a = fabs(v);
    return a != a ? 0.0 : a;
}

/* Algorithm 1, the two per-map quantities: for the map dY[n,k,:,:]
 *   idx = flat position h*Wo + w of the largest |dY|; the scan runs over
 *         ascending flat position with a strict '>' so the lowest position wins
 *         ties; +v and -v have equal magnitude; an all-zero map gives 0; a NaN
 *         ranks as a zero (see rank_magnitude);
 *   S   = the signed sum of the whole map, a scalar. */
static void select_map(const double *map, int len, int32_t *idx, double *S)
{
    double best = -1.0, sum = 0.0;
    int32_t where = 0;
    for (int p = 0; p < len; ++p) {
        double a = rank_magnitude(map[p]);
        if (a > best) { best = a; where = p; }
        sum += map[p];
    }
    *idx = where;
    *S = sum;
}

/* idx[n*K + k], S[n*K + k] for every map. */
int oracle_select(const oracle_shape *g, const void *dY_, int dtype, int32_t *idx, double *S)
{
    const int Ho = out_h(g), Wo = out_w(g), len = Ho * Wo;
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * len);
    if (!dY) return -1;
    const long maps = (long)g->N * g->K;
#pragma omp parallel for schedule(static)
    for (long m = 0; m < maps; ++m) select_map(dY + (size_t)m * len, len, &idx[m], &S[m]);
    free(dY);
    return 0;
}

/* Algorithm 1 (Max Gradient Approximation), in the paper's loop order:
 *   dW = 0
 *   for each output channel k, for each batch element n:
 *       (row, col) = argmax |dY[n,k,:,:]| ;  sum = sum of dY[n,k,:,:]
 *       dW[k,:,:,:] += patch of X[n] anchored at (row, col) * sum
 *   dW *= scale        (Section 2.3 scales the result by a constant; 1 = as printed)
 * The patch element (c,r,s) is X[n,c,row*stride_h + r - pad_h, col*stride_w + s - pad_w]
 * with zero outside X, i.e. exactly the input element that output position
 * (row,col) sees through filter tap (r,s); with that reading the approximation
 * equals the exact gradient of the sparsified dY for padded and strided layers.
 * idx_out / S_out (each N*K, may be NULL) receive the per-map selections. */
int oracle_wgrad_approx(const oracle_shape *g, const void *X_, const void *dY_, int dtype,
                        double scale, double *dW, int32_t *idx_out, double *S_out)
{
    const int Ho = out_h(g), Wo = out_w(g), len = Ho * Wo;
    double *X = to_double(X_, dtype, (size_t)g->N * g->C * g->H * g->W);
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * len);
    if (!X || !dY) { free(X); free(dY); return -1; }
    const size_t per_k = (size_t)g->C * g->R * g->S;
    for (size_t o = 0; o < per_k * g->K; ++o) dW[o] = 0.0;
#pragma omp parallel for schedule(static)
    for (int k = 0; k < g->K; ++k) {
        for (int n = 0; n < g->N; ++n) {
            int32_t where; double sum;
            select_map(dY + ((size_t)n * g->K + k) * len, len, &where, &sum);
            if (idx_out) idx_out[(size_t)n * g->K + k] = where;
            if (S_out) S_out[(size_t)n * g->K + k] = sum;
            const int row = where / Wo, col = where % Wo;
            for (int c = 0; c < g->C; ++c)
                for (int r = 0; r < g->R; ++r)
                    for (int s = 0; s < g->S; ++s)
                        dW[k * per_k + ((size_t)c * g->R + r) * g->S + s] +=
                            x_at(X, g, n, c, row * g->stride_h + r - g->pad_h,
                                 col * g->stride_w + s - g->pad_w) * sum;
        }
        for (size_t o = 0; o < per_k; ++o) dW[k * per_k + o] *= scale;
    }
    free(X); free(dY);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Top-k generalisation (Section 2.3 names it in one sentence -- keep the k
 * largest-magnitude values of a map "with an adjustment of the scaling
 * parameter" -- and leaves the adjustment open).  Reading used by this build:
 * the k retained positions of a map each carry sum/k, so that k = 1 is
 * Algorithm 1 and the total weight of a map stays its sum.  Positions are taken
 * in order of decreasing magnitude, equal magnitudes by increasing flat index;
 * k is clamped to the map length.
 * idx[(n*K + k_out)*k + j] = j-th retained position, S[n*K + k_out] = map sum.
 * ------------------------------------------------------------------------- */
static void select_map_topk(const double *map, int len, int k, int32_t *where, double *sum)
{
    double s = 0.0;
    for (int p = 0; p < len; ++p) s += map[p];
    *sum = s;
    /* k passes, each a first-maximum scan over the positions not taken yet */
    for (int j = 0; j < k; ++j) {
        double best = -1.0;
        int at = 0;
        for (int p = 0; p < len; ++p) {
            int taken = 0;
            for (int i = 0; i < j; ++i) taken |= where[i] == p;
            if (taken) continue;
            const double a = rank_magnitude(map[p]);
            if (a > best) { best = a; at = p; }
        }
        where[j] = at;
    }
}

int oracle_select_topk(const oracle_shape *g, const void *dY_, int dtype, int k, int32_t *idx, double *S)
{
    const int Ho = out_h(g), Wo = out_w(g), len = Ho * Wo;
    if (k < 1 || k > len) return -2;
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * len);
    if (!dY) return -1;
    const long maps = (long)g->N * g->K;
#pragma omp parallel for schedule(static)
    for (long m = 0; m < maps; ++m) select_map_topk(dY + (size_t)m * len, len, k, idx + (size_t)m * k, &S[m]);
    free(dY);
    return 0;
}

int oracle_wgrad_approx_topk(const oracle_shape *g, const void *X_, const void *dY_, int dtype, int k,
                             double scale, double *dW, int32_t *idx_out, double *S_out)
{
    const int Ho = out_h(g), Wo = out_w(g), len = Ho * Wo;
    if (k < 1 || k > len || k > 64) return -2;
    double *X = to_double(X_, dtype, (size_t)g->N * g->C * g->H * g->W);
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * len);
    if (!X || !dY) { free(X); free(dY); return -1; }
    const size_t per_k = (size_t)g->C * g->R * g->S;
    for (size_t o = 0; o < per_k * g->K; ++o) dW[o] = 0.0;
#pragma omp parallel for schedule(static)
    for (int ko = 0; ko < g->K; ++ko) {
        for (int n = 0; n < g->N; ++n) {
            int32_t where[64]; double sum;
            select_map_topk(dY + ((size_t)n * g->K + ko) * len, len, k, where, &sum);
            if (S_out) S_out[(size_t)n * g->K + ko] = sum;
            const double share = sum / k;
            for (int j = 0; j < k; ++j) {
                if (idx_out) idx_out[((size_t)n * g->K + ko) * k + j] = where[j];
                const int row = where[j] / Wo, col = where[j] % Wo;
                for (int c = 0; c < g->C; ++c)
                    for (int r = 0; r < g->R; ++r)
                        for (int s = 0; s < g->S; ++s)
                            dW[ko * per_k + ((size_t)c * g->R + r) * g->S + s] +=
                                x_at(X, g, n, c, row * g->stride_h + r - g->pad_h,
                                     col * g->stride_w + s - g->pad_w) * share;
            }
        }
        for (size_t o = 0; o < per_k; ++o) dW[ko * per_k + o] *= scale;
    }
    free(X); free(dY);
    return 0;
}

/* ---------------------------------------------------------------------------
 * The layouts of the paper's own kernel (Section 2.4, last paragraphs):
 * input activations channel-last, X[n,h,w,c]; output gradient unchanged,
 * dY[n,k,h,w]; filter gradient produced as [C_o,K,K,C_i] = dW[k,r,s,c]
 * ("OHWI"), and afterwards transposed to the [K,K,C_i,C_o] = dW[r,s,c,k]
 * ("HWIO") form in which Section 2.4 writes the filter tensor.  The values are
 * those of the definitions above; only where an element lives changes.  These
 * functions index the channel-last tensors directly, they do not go through
 * the NCHW functions (the tests compare the two routes).
 * ------------------------------------------------------------------------- */
enum { ORACLE_DW_OIHW = 0, ORACLE_DW_OHWI = 1, ORACLE_DW_HWIO = 2 };

static double x_at_nhwc(const double *X, const oracle_shape *g, int n, int ih, int iw, int c)
{
    if (ih < 0 || ih >= g->H || iw < 0 || iw >= g->W) return 0.0;
    return X[(((size_t)n * g->H + ih) * g->W + iw) * g->C + c];
}

/* where dW(k,c,r,s) lives in a filter-gradient tensor of the given layout */
static size_t dw_offset(const oracle_shape *g, int layout, int k, int c, int r, int s)
{
    if (layout == ORACLE_DW_OHWI) return (((size_t)k * g->R + r) * g->S + s) * g->C + c;
    if (layout == ORACLE_DW_HWIO) return (((size_t)r * g->S + s) * g->C + c) * g->K + k;
    return (((size_t)k * g->C + c) * g->R + r) * g->S + s;
}

int oracle_wgrad_exact_nhwc(const oracle_shape *g, const void *X_, const void *dY_, int dtype,
                            int dw_layout, double *dW)
{
    const int Ho = out_h(g), Wo = out_w(g);
    double *X = to_double(X_, dtype, (size_t)g->N * g->C * g->H * g->W);
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * Ho * Wo);
    if (!X || !dY) { free(X); free(dY); return -1; }
#pragma omp parallel for schedule(static) collapse(2)
    for (int k = 0; k < g->K; ++k)
        for (int c = 0; c < g->C; ++c)
            for (int r = 0; r < g->R; ++r)
                for (int s = 0; s < g->S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < g->N; ++n)
                        for (int h = 0; h < Ho; ++h)
                            for (int w = 0; w < Wo; ++w)
                                acc += dY[(((size_t)n * g->K + k) * Ho + h) * Wo + w] *
                                       x_at_nhwc(X, g, n, h * g->stride_h + r - g->pad_h,
                                                 w * g->stride_w + s - g->pad_w, c);
                    dW[dw_offset(g, dw_layout, k, c, r, s)] = acc;
                }
    free(X); free(dY);
    return 0;
}

/* Algorithm 1 on the channel-last input: the patch of map (n,k) is the R x S x C
 * block of X[n] whose corner is the selected position (its C values per tap are
 * contiguous, which is why the paper's kernel wants this layout). */
int oracle_wgrad_approx_nhwc(const oracle_shape *g, const void *X_, const void *dY_, int dtype,
                             int dw_layout, double scale, double *dW, int32_t *idx_out, double *S_out)
{
    const int Ho = out_h(g), Wo = out_w(g), len = Ho * Wo;
    double *X = to_double(X_, dtype, (size_t)g->N * g->C * g->H * g->W);
    double *dY = to_double(dY_, dtype, (size_t)g->N * g->K * len);
    if (!X || !dY) { free(X); free(dY); return -1; }
    const size_t total = (size_t)g->K * g->C * g->R * g->S;
    for (size_t o = 0; o < total; ++o) dW[o] = 0.0;
#pragma omp parallel for schedule(static)
    for (int k = 0; k < g->K; ++k) {
        for (int n = 0; n < g->N; ++n) {
            int32_t where; double sum;
            select_map(dY + ((size_t)n * g->K + k) * len, len, &where, &sum);
            if (idx_out) idx_out[(size_t)n * g->K + k] = where;
            if (S_out) S_out[(size_t)n * g->K + k] = sum;
            const int row = where / Wo, col = where % Wo;
            for (int r = 0; r < g->R; ++r)
                for (int s = 0; s < g->S; ++s)
                    for (int c = 0; c < g->C; ++c)
                        dW[dw_offset(g, dw_layout, k, c, r, s)] +=
                            x_at_nhwc(X, g, n, row * g->stride_h + r - g->pad_h,
                                      col * g->stride_w + s - g->pad_w, c) * sum;
        }
        for (int r = 0; r < g->R; ++r)
            for (int s = 0; s < g->S; ++s)
                for (int c = 0; c < g->C; ++c) dW[dw_offset(g, dw_layout, k, c, r, s)] *= scale;
    }
    free(X); free(dY);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Random gradient (Section 2.2): independent N(0, sigma) values, new for every
 * batch.  The paper drew them on the host with a library generator; what the
 * method fixes is the distribution only.  This build defines the stream as a
 * pure function of (seed, offset + i) so the GPU can be checked value by value.
 * One Philox call gives four 32-bit words, i.e. two Box-Muller pairs, i.e. four
 * independent normals (the cosine and the sine of one pair are independent), so
 * four consecutive stream positions share a call:
 *   g = offset + i,  c = g / 4,  j = g mod 4
 *   (w0,w1,w2,w3) = Philox4x32-10(counter = (lo32(c), hi32(c), 0, 0),
 *                                 key = (lo32(seed), hi32(seed)))
 *   pair p = j / 2:  u1 = ((w[2p] >> 8) + 0.5) / 2^24,  u2 = ((w[2p+1] >> 8) + 0.5) / 2^24   (both in (0,1))
 *   value = sigma * sqrt(-2 ln u1) * (j even ? cos(2 pi u2) : sin(2 pi u2))                    (Box-Muller)
 * Philox4x32-10 is the counter-based generator of Salmon, Moraes, Dror and
 * Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11).
 * ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4])
{
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void oracle_random_normal(uint64_t seed, uint64_t offset, int64_t count, double sigma, double *out)
{
    const double two_pi = 6.283185307179586476925286766559;
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t i = 0; i < count; ++i) {
        uint64_t gidx = offset + (uint64_t)i;
        uint64_t c = gidx >> 2;
        int j = (int)(gidx & 3u);
        uint32_t ctr[4] = { (uint32_t)c, (uint32_t)(c >> 32), 0u, 0u };
        uint32_t w[4];
        oracle_philox4x32_10(ctr, key, w);
        int p = j >> 1;
        double u1 = ((double)(w[2 * p] >> 8) + 0.5) / 16777216.0;
        double u2 = ((double)(w[2 * p + 1] >> 8) + 0.5) / 16777216.0;
        double radius = sqrt(-2.0 * log(u1));
        out[i] = sigma * radius * ((j & 1) ? sin(two_pi * u2) : cos(two_pi * u2));
    }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
